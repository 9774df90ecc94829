"""Input generators (numpy Philox streams; every draw is a function of the seed only)."""
from dataclasses import dataclass, field
import numpy as np

SEED0 = 0x13779


def rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def to_bf16_bits(f32: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round-to-nearest-even.  Finite inputs only."""
    u = np.ascontiguousarray(f32, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def normal_bf16(g: np.random.Generator, shape, std: float) -> np.ndarray:
    """N(0, std^2) drawn in float32, stored as bf16 bits."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        out[lo:hi] = to_bf16_bits(g.standard_normal(hi - lo, dtype=np.float32) * np.float32(std))
    return out.reshape(shape)


def zipf_slots(g: np.random.Generator, T: int, n_slots: int, s: float) -> np.ndarray:
    """P(slot = k-1) proportional to k^-s, k = 1..n_slots, by inverse CDF on a uniform stream."""
    w = np.arange(1, n_slots + 1, dtype=np.float64) ** (-s)
    cdf = np.cumsum(w / w.sum())
    u = g.random(T)
    return np.minimum(np.searchsorted(cdf, u, side="right"), n_slots - 1).astype(np.int32)


def lognormal_segments(g: np.random.Generator, T: int, S: int, mu: float, sigma: float) -> np.ndarray:
    """S lengths ~ exp(mu + sigma z), renormalised to integers >= 1 summing to T
    (largest-remainder rounding, ties to the lower index).  Returns offsets [S+1]."""
    ell = np.exp(mu + sigma * g.standard_normal(S))
    share = T * ell / ell.sum()
    L = np.floor(share).astype(np.int64)
    L = np.maximum(L, 1)
    rem = T - int(L.sum())
    frac = share - np.floor(share)
    order = sorted(range(S), key=lambda k: (-frac[k], k))
    i = 0
    while rem > 0:
        L[order[i % S]] += 1
        rem -= 1
        i += 1
    while rem < 0:  # only if the >= 1 clamp overshot
        k = int(np.argmax(L))
        L[k] -= 1
        rem += 1
    off = np.zeros(S + 1, dtype=np.int32)
    off[1:] = np.cumsum(L)
    assert off[-1] == T and (L >= 1).all()
    return off


def topk_routing(g: np.random.Generator, T: int, E: int, K: int) -> np.ndarray:
    """Top-K experts of N(0,1) logits per token (softmax is monotone, so top-K of the logits),
    listed in descending-logit order, ties to the lower expert id.  int32 [T, K]."""
    logits = g.standard_normal((T, E), dtype=np.float32)
    order = np.argsort(-logits, axis=1, kind="stable")
    return np.ascontiguousarray(order[:, :K]).astype(np.int32)


@dataclass
class DenseCase:
    """One dense LoRA site and one decode batch for it.  A is [S, r_max, d_in], B is
    [S, d_out, r_max] (rows/columns >= rank[s] are zero)."""
    name: str
    T: int
    d_in: int
    d_out: int
    n_slots: int
    r_max: int
    x: np.ndarray
    y0: np.ndarray
    A: np.ndarray
    B: np.ndarray
    rank: np.ndarray
    alpha: np.ndarray
    token_slot: np.ndarray
    catalog_id: np.ndarray = field(default=None)


@dataclass
class SegCase(DenseCase):
    seg_off: np.ndarray = field(default=None)
    seg_slot: np.ndarray = field(default=None)


@dataclass
class MoECase:
    """Packed MoE site: A [S, E, r_max, d_in], B [S, E, d_out, r_max]; y0 is pair-major [T*K, d_out]."""
    name: str
    T: int
    K: int
    E: int
    d_in: int
    d_out: int
    n_slots: int
    r_max: int
    x: np.ndarray
    y0: np.ndarray
    A: np.ndarray
    B: np.ndarray
    rank: np.ndarray
    alpha: np.ndarray
    token_slot: np.ndarray
    topk: np.ndarray


@dataclass
class MoEDownCase:
    """Packed MoE site on the expert down projection: x is pair-major [T*K, d_in] (an expert's
    intermediate activation per routed pair), y0 is token-major [T, d_out], w [T, K] fp32 routing
    weights (positive, summing to one per token)."""
    name: str
    T: int
    K: int
    E: int
    d_in: int
    d_out: int
    n_slots: int
    r_max: int
    x: np.ndarray
    y0: np.ndarray
    A: np.ndarray
    B: np.ndarray
    rank: np.ndarray
    alpha: np.ndarray
    token_slot: np.ndarray
    topk: np.ndarray
    w: np.ndarray


def _adapters(g, lead, r_max, d_in, d_out, ranks_per_slot, std_a, std_b):
    """lead = (S,) or (S, E).  Rows j >= rank of the slot are zero-filled."""
    A = normal_bf16(g, lead + (r_max, d_in), std_a)
    B = normal_bf16(g, lead + (d_out, r_max), std_b)
    for s, r in enumerate(ranks_per_slot):
        if r < r_max:
            A[s, ..., r:, :] = 0
            B[s, ..., :, r:] = 0
    return A, B


def dense_case(name, seed, T, d_in, d_out, n_slots, r_max, alpha, *, ranks=None,
               std_x=1.0, std_y=1.0, std_a=0.02, std_b=0.02, token_slot=None) -> DenseCase:
    g = rng(seed)
    ranks = np.full(n_slots, r_max, dtype=np.int32) if ranks is None else np.asarray(ranks, dtype=np.int32)
    x = normal_bf16(g, (T, d_in), std_x)
    y0 = normal_bf16(g, (T, d_out), std_y)
    A, B = _adapters(g, (n_slots,), r_max, d_in, d_out, ranks, std_a, std_b)
    if token_slot is None:
        token_slot = g.integers(-1, n_slots, size=T).astype(np.int32)
    alpha_arr = np.broadcast_to(np.asarray(alpha, dtype=np.float64), (n_slots,)).copy()
    cat = g.permutation(10 ** 6)[:n_slots].astype(np.int64)
    return DenseCase(name, T, d_in, d_out, n_slots, r_max, x, y0, A, B, ranks, alpha_arr,
                     np.asarray(token_slot, dtype=np.int32), cat)


def seg_case(name, seed, T, S, d_in, d_out, n_slots, r_max, alpha, *, mu=6.0, sigma=0.8,
             ranks=None, seg_off=None, seg_slot=None, std_x=1.0, std_y=1.0,
             std_a=0.02, std_b=0.02) -> SegCase:
    g = rng(seed)
    ranks = np.full(n_slots, r_max, dtype=np.int32) if ranks is None else np.asarray(ranks, dtype=np.int32)
    if seg_off is None:
        seg_off = lognormal_segments(g, T, S, mu, sigma)
    seg_off = np.asarray(seg_off, dtype=np.int32)
    if seg_slot is None:
        seg_slot = g.integers(0, n_slots, size=S).astype(np.int32)
    seg_slot = np.asarray(seg_slot, dtype=np.int32)
    x = normal_bf16(g, (T, d_in), std_x)
    y0 = normal_bf16(g, (T, d_out), std_y)
    A, B = _adapters(g, (n_slots,), r_max, d_in, d_out, ranks, std_a, std_b)
    token_slot = np.repeat(seg_slot, np.diff(seg_off)).astype(np.int32)
    alpha_arr = np.broadcast_to(np.asarray(alpha, dtype=np.float64), (n_slots,)).copy()
    return SegCase(name, T, d_in, d_out, n_slots, r_max, x, y0, A, B, ranks, alpha_arr,
                   token_slot, None, seg_off, seg_slot)


def moe_case(name, seed, T, K, E, d_in, d_out, n_slots, r_max, alpha, *, ranks=None,
             token_slot=None, std_x=1.0, std_y=1.0, std_a=0.02, std_b=0.02) -> MoECase:
    g = rng(seed)
    ranks = np.full(n_slots, r_max, dtype=np.int32) if ranks is None else np.asarray(ranks, dtype=np.int32)
    x = normal_bf16(g, (T, d_in), std_x)
    y0 = normal_bf16(g, (T * K, d_out), std_y)
    A, B = _adapters(g, (n_slots, E), r_max, d_in, d_out, ranks, std_a, std_b)
    if token_slot is None:
        token_slot = g.integers(0, n_slots, size=T).astype(np.int32)
    topk = topk_routing(g, T, E, K)
    alpha_arr = np.broadcast_to(np.asarray(alpha, dtype=np.float64), (n_slots,)).copy()
    return MoECase(name, T, K, E, d_in, d_out, n_slots, r_max, x, y0, A, B, ranks, alpha_arr,
                   np.asarray(token_slot, dtype=np.int32), topk)


# ---- the five benchmark configurations ------------------------------------------------------

def routing_weights(g: np.random.Generator, T: int, K: int) -> np.ndarray:
    """Softmax over K N(0,1) logits per token (the weights of the selected experts renormalised
    over the selection), fp32 [T, K]."""
    z = g.standard_normal((T, K), dtype=np.float32).astype(np.float64)
    e = np.exp(z - z.max(axis=1, keepdims=True))
    return np.ascontiguousarray((e / e.sum(axis=1, keepdims=True)).astype(np.float32))


def moe_down_case(name, seed, T, K, E, d_in, d_out, n_slots, r_max, alpha, *, ranks=None,
                  token_slot=None, std_x=1.0, std_y=1.0, std_a=0.02, std_b=0.02) -> MoEDownCase:
    g = rng(seed)
    ranks = np.full(n_slots, r_max, dtype=np.int32) if ranks is None else np.asarray(ranks, dtype=np.int32)
    x = normal_bf16(g, (T * K, d_in), std_x)
    y0 = normal_bf16(g, (T, d_out), std_y)
    A, B = _adapters(g, (n_slots, E), r_max, d_in, d_out, ranks, std_a, std_b)
    if token_slot is None:
        token_slot = g.integers(0, n_slots, size=T).astype(np.int32)
    topk = topk_routing(g, T, E, K)
    w = routing_weights(g, T, K)
    alpha_arr = np.broadcast_to(np.asarray(alpha, dtype=np.float64), (n_slots,)).copy()
    return MoEDownCase(name, T, K, E, d_in, d_out, n_slots, r_max, x, y0, A, B, ranks, alpha_arr,
                       np.asarray(token_slot, dtype=np.int32), topk, w)


def c1_tiny_decode() -> DenseCase:
    """64 tokens, 256->256, 8 slots rank 8 alpha 16, values ~N(0, 1/sqrt(fan_in)) (fan_in = d_in
    for x, A and y0; = r for B), slot index uniform in {-1..7}."""
    d, r = 256, 8
    return dense_case("c1_tiny", SEED0 + 1, 64, d, d, 8, r, 16.0,
                      std_x=d ** -0.5, std_y=d ** -0.5, std_a=d ** -0.5, std_b=r ** -0.5)


c2_projections = (
    ("q", 2560, 2560), ("k", 2560, 1024), ("v", 2560, 1024), ("o", 2560, 2560),
    ("gate", 2560, 9728), ("up", 2560, 9728), ("down", 9728, 2560),
)


def c2_dense_decode(layer: int = 0):
    """One layer of the 4B-dense-like decode: 256 tokens, seven projections, 64 slots rank 16
    alpha 32, adapters ~N(0, 0.02), slot per token Zipf(1.1).  All seven sites share the batch's
    token->slot map.  Returns a list of DenseCase."""
    T, S, r = 256, 64, 16
    slots = zipf_slots(rng(SEED0 + 2), T, S, 1.1)
    out = []
    for i, (nm, d_in, d_out) in enumerate(c2_projections):
        out.append(dense_case(f"c2_{nm}", SEED0 + 200 + 16 * layer + i, T, d_in, d_out, S, r, 32.0,
                              token_slot=slots))
    return out


def c3_rank1_catalog() -> DenseCase:
    """512 decode tokens, 4096->4096, 1024 resident rank-1 slots (alpha 1) paged in from a
    10^6-entry catalog id space; every token has its own slot."""
    T, S = 512, 1024
    slots = rng(SEED0 + 3).permutation(S)[:T].astype(np.int32)
    return dense_case("c3_rank1", SEED0 + 300, T, 4096, 4096, S, 1, 1.0, token_slot=slots)


def c4_moe_packed(proj: str = "gate") -> MoECase:
    """2048 tokens, hidden 2048, 128 experts of intermediate 768, top-8, 32 slots rank 8
    alpha 16; gate and up are two sites over the same routing."""
    i = {"gate": 0, "up": 1}[proj]
    c = moe_case(f"c4_{proj}", SEED0 + 400 + i, 2048, 8, 128, 2048, 768, 32, 8, 16.0)
    g = rng(SEED0 + 4)  # routing and slots are shared by both projections
    c.token_slot = g.integers(0, 32, size=2048).astype(np.int32)
    c.topk = topk_routing(g, 2048, 128, 8)
    return c


def c4_moe_mixed_rank() -> MoECase:
    """The gate site of the c4 layer with heterogeneous adapters (ranks differ between the tenants
    of one worker and are padded into the shape of the largest one): each of the 32 slots draws its
    rank from {2, 4, 8} with equal probability, alpha = 2 * rank; tables of rank 8; same routing
    and slots as c4."""
    g = rng(SEED0 + 4)
    token_slot = g.integers(0, 32, size=2048).astype(np.int32)
    topk = topk_routing(g, 2048, 128, 8)
    ranks = rng(SEED0 + 44).choice(np.array([2, 4, 8], dtype=np.int32), size=32)
    c = moe_case("c4_mixed", SEED0 + 404, 2048, 8, 128, 2048, 768, 32, 8, 2.0 * ranks, ranks=ranks)
    c.token_slot, c.topk = token_slot, topk
    return c


def c4_moe_down() -> MoEDownCase:
    """The down projection of the c4 layer: 2048 tokens, 128 experts of intermediate 768 back to
    hidden 2048, top-8 with routing weights, 32 slots rank 8 alpha 16; routing and slots are the
    ones of the gate and up sites."""
    c = moe_down_case("c4_down", SEED0 + 402, 2048, 8, 128, 768, 2048, 32, 8, 16.0)
    g = rng(SEED0 + 4)
    c.token_slot = g.integers(0, 32, size=2048).astype(np.int32)
    c.topk = topk_routing(g, 2048, 128, 8)
    return c


def c5_segmented(wide: bool = False) -> SegCase:
    """8192 tokens in 16 lognormal(6, 0.8) segments, 16 slots rank 64 alpha 128,
    7168->7168 (or 7168->18432 with wide=True)."""
    d_out = 18432 if wide else 7168
    g = rng(SEED0 + 5)
    seg_off = lognormal_segments(g, 8192, 16, 6.0, 0.8)
    seg_slot = g.integers(0, 16, size=16).astype(np.int32)
    return seg_case("c5_wide" if wide else "c5", SEED0 + 500 + int(wide), 8192, 16, 7168, d_out,
                    16, 64, 128.0, seg_off=seg_off, seg_slot=seg_slot)
