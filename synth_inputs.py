"""Seeded synthetic inputs for the Amphista draft+verify hot path.

This module only *generates data*: configurations, random weights, hidden
states, token ids, KV caches and candidate-tree topologies (as lists of rank
paths).  It holds none of the method's arithmetic, so both the CPU oracle's
tests and the HIP path's tests/bench may import it without sharing any
computation between the two sides.

Every tensor comes from numpy.random.default_rng(SeedSequence([seed, config_id,
crc32(name)])) on the host.  In bf16 configurations a tensor is rounded to
bf16 (round-to-nearest-even) exactly once here; the oracle receives the widened
float32 values and the GPU receives the same 16-bit patterns.

The shapes stand in for the paper's Vicuna 7B/13B/33B targets with K = 4 (5)
drafting heads and a 64 (96) node draft tree (Experimental Settings; Appendix
"Draft Tree"); values are a neutral N(0, 0.02^2) / N(0, 1) stand-in for the
trained weights and benchmark prompts, which are not available.
"""
from __future__ import annotations

import heapq
import zlib
from dataclasses import dataclass, replace
from typing import Dict, List, Sequence, Tuple

import numpy as np

F32 = "f32"
BF16 = "bf16"


@dataclass(frozen=True)
class Config:
    name: str
    config_id: int
    d_model: int
    n_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_layers: int          # target decoder layers
    K: int                 # drafting heads
    topk: int              # per-head top-k
    T: int                 # tree nodes incl. root
    kv_len: int            # committed target KV rows before the step (L)
    sal_len: int           # committed rows in each SAL cache (L_s)
    batch: int
    dtype: str
    tree_caps: Tuple[int, ...]
    rms_eps: float = 1e-6
    rope_theta: float = 10000.0
    n_stages: int = 2

    @property
    def max_kv(self) -> int:
        """Cache capacity: room for the tree rows, rounded up to 32 rows."""
        need = max(self.kv_len + self.T, self.sal_len + 1)
        return (need + 31) // 32 * 32


TINY = Config("tiny", 1, 256, 4, 64, 688, 1024, 2, 4, 4, 16, 128, 128, 1, F32, (4, 2, 2, 2))
V7B = Config("vicuna7b", 2, 4096, 32, 128, 11008, 32000, 32, 4, 10, 64, 1024, 1024, 1, BF16,
             (10, 10, 10, 10))
V13B = Config("vicuna13b", 4, 5120, 40, 128, 13824, 32000, 40, 4, 10, 64, 2048, 2048, 1, BF16,
              (10, 10, 10, 10))
V33B = Config("vicuna33b", 5, 6656, 52, 128, 17920, 32000, 60, 5, 10, 96, 4096, 4096, 4, BF16,
              (10, 10, 10, 10, 10))
# A bf16 miniature with 128-wide heads: several tiles and ragged tails at a size
# the oracle finishes in seconds.
MINI = Config("mini_bf16", 6, 512, 4, 128, 1376, 2048, 2, 4, 10, 64, 200, 77, 1, BF16,
              (10, 10, 10, 10))

CONFIGS = {c.name: c for c in (TINY, V7B, V13B, V33B, MINI)}


def with_(cfg: Config, **kw) -> Config:
    return replace(cfg, **kw)


# ----------------------------------------------------------------------------
# bf16 bit handling (data preparation only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest even), return the uint16 patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class Tensor:
    """One synthetic tensor: `f32` is what the oracle sees, `dev` what the GPU gets.

    For bf16 configurations `dev` is a uint16 array of bf16 patterns and `f32`
    the same values widened; for f32 configurations both are the same array.
    """
    f32: np.ndarray
    dev: np.ndarray
    dtype: str


def _rng(cfg: Config, seed: int, name: str) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([seed, cfg.config_id, zlib.crc32(name.encode())]))


def normal(cfg: Config, seed: int, name: str, shape: Sequence[int], std: float,
           dtype: str | None = None) -> Tensor:
    dtype = dtype or cfg.dtype
    a = _rng(cfg, seed, name).standard_normal(tuple(shape), dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if dtype == BF16:
        bits = f32_to_bf16_bits(a)
        return Tensor(bf16_bits_to_f32(bits), bits, BF16)
    return Tensor(a, a, F32)


def ones(cfg: Config, shape: Sequence[int], dtype: str | None = None) -> Tensor:
    dtype = dtype or cfg.dtype
    a = np.ones(tuple(shape), dtype=np.float32)
    if dtype == BF16:
        bits = f32_to_bf16_bits(a)
        return Tensor(a, bits, BF16)
    return Tensor(a, a, F32)


def as_f32_exact(cfg: Config, seed: int, name: str, shape: Sequence[int], std: float) -> np.ndarray:
    """float32 activations whose values are exactly representable in cfg.dtype."""
    return normal(cfg, seed, name, shape, std).f32.copy()


def tokens(cfg: Config, seed: int, name: str, shape: Sequence[int]) -> np.ndarray:
    return _rng(cfg, seed, name).integers(0, cfg.vocab, size=tuple(shape), dtype=np.int32)


# ----------------------------------------------------------------------------
# weight bundles
# ----------------------------------------------------------------------------
W_STD = 0.02
LAYER_KEYS = ("rms1", "wq", "wk", "wv", "wo", "rms2", "w_gate", "w_up", "w_down")


def decoder_layer(cfg: Config, seed: int, prefix: str) -> Dict[str, Tensor]:
    d, f = cfg.d_model, cfg.d_ffn
    n = lambda nm, shp: normal(cfg, seed, f"{prefix}.{nm}", shp, W_STD)
    return {
        "rms1": ones(cfg, (d,)), "rms2": ones(cfg, (d,)),
        "wq": n("wq", (d, d)), "wk": n("wk", (d, d)), "wv": n("wv", (d, d)), "wo": n("wo", (d, d)),
        "w_gate": n("w_gate", (f, d)), "w_up": n("w_up", (f, d)), "w_down": n("w_down", (d, f)),
    }


def draft_weights(cfg: Config, seed: int = 0) -> Dict[str, object]:
    """Embed table, fc^1/fc^2, SAL^1/SAL^2, K head MLPs, PE, self-attention, shared LM head."""
    d, V, K = cfg.d_model, cfg.vocab, cfg.K
    n = lambda nm, shp: normal(cfg, seed, f"draft.{nm}", shp, W_STD)
    return {
        "embed": normal(cfg, seed, "target.embed", (V, d), W_STD),
        "fc": [n(f"fc{s}", (d, 2 * d)) for s in range(cfg.n_stages)],
        "sal": [decoder_layer(cfg, seed, f"draft.sal{s}") for s in range(cfg.n_stages)],
        "mlp": n("mlp", (K, d, d)),
        "pe": n("pe", (K, d)),
        "aeb_wq": n("aeb_wq", (d, d)), "aeb_wk": n("aeb_wk", (d, d)),
        "aeb_wv": n("aeb_wv", (d, d)), "aeb_wo": n("aeb_wo", (d, d)),
        "lm_head": n("lm_head", (V, d)),
    }


def target_weights(cfg: Config, seed: int = 0, n_layers: int | None = None) -> Dict[str, object]:
    d, V = cfg.d_model, cfg.vocab
    nl = cfg.n_layers if n_layers is None else n_layers
    return {
        "embed": normal(cfg, seed, "target.embed", (V, d), W_STD),
        "layers": [decoder_layer(cfg, seed, f"target.layer{i}") for i in range(nl)],
        "final_norm": ones(cfg, (d,)),
        "lm_head": normal(cfg, seed, "target.lm_head", (V, d), W_STD),
    }


def kv_cache_rows(cfg: Config, seed: int, name: str, rows: int) -> Tuple[Tensor, Tensor]:
    """Committed K and V rows [B, n_heads, rows, head_dim] ~ N(0,1) (keys are post-RoPE,
    so any values are valid cache contents)."""
    shp = (cfg.batch, cfg.n_heads, rows, cfg.head_dim)
    return normal(cfg, seed, name + ".k", shp, 1.0), normal(cfg, seed, name + ".v", shp, 1.0)


# ----------------------------------------------------------------------------
# candidate-tree topology (rank paths).  Integer-only best-first generator that
# stands in for the paper's dataset-tuned tree (Appendix "Draft Tree"): a path's
# cost is sum(rank + 1); nodes are added in increasing (cost, depth, path) order.
# ----------------------------------------------------------------------------
def tree_paths(T: int, caps: Sequence[int]) -> List[Tuple[int, ...]]:
    """Return T-1 rank paths (the root is implicit), each a tuple of length 1..len(caps)."""
    K = len(caps)
    out: List[Tuple[int, ...]] = []
    heap: List[Tuple[int, int, Tuple[int, ...]]] = []
    if T > 1 and K > 0 and caps[0] > 0:
        heapq.heappush(heap, (1, 1, (0,)))
    while heap and len(out) < T - 1:
        cost, depth, path = heapq.heappop(heap)
        out.append(path)
        r = path[-1]
        if r + 1 < caps[depth - 1]:
            heapq.heappush(heap, (cost + 1, depth, path[:-1] + (r + 1,)))
        if depth < K and caps[depth] > 0:
            heapq.heappush(heap, (cost + 1, depth + 1, path + (0,)))
    if len(out) != T - 1:
        raise ValueError("caps too small for the requested tree size")
    return out


def random_tree_paths(T: int, K: int, topk: int, seed: int) -> List[Tuple[int, ...]]:
    """T-1 rank paths of an irregular tree: every new node hangs under a random existing node of depth < K
    that still has an unused rank below topk, with a random unused rank (siblings' ranks need not be
    contiguous).  Order of the list is the order of creation, i.e. not sorted."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, T, K, topk, 0x7ee]))
    nodes: List[Tuple[int, ...]] = [()]
    used = {(): set()}
    while len(nodes) < T:
        open_nodes = [p for p in nodes if len(p) < K and len(used[p]) < topk]
        if not open_nodes:
            raise ValueError("no room left for another node")
        par = open_nodes[int(rng.integers(0, len(open_nodes)))]
        free = [r for r in range(topk) if r not in used[par]]
        r = free[int(rng.integers(0, len(free)))]
        used[par].add(r)
        child = par + (r,)
        nodes.append(child)
        used[child] = set()
    return nodes[1:]


def dense_tree_paths(widths: Sequence[int]) -> List[Tuple[int, ...]]:
    """Full tree: every node at depth j-1 has widths[j-1] children."""
    level: List[Tuple[int, ...]] = [()]
    out: List[Tuple[int, ...]] = []
    for w in widths:
        nxt = [p + (r,) for p in level for r in range(w)]
        out += nxt
        level = nxt
    return out


def chain_tree_paths(K: int) -> List[Tuple[int, ...]]:
    return [tuple([0] * m) for m in range(1, K + 1)]


def star_tree_paths(n: int) -> List[Tuple[int, ...]]:
    return [(r,) for r in range(n)]


def paths_to_array(paths: Sequence[Sequence[int]], K: int) -> np.ndarray:
    a = np.full((len(paths), K), -1, dtype=np.int32)
    for i, p in enumerate(paths):
        a[i, :len(p)] = p
    return a
