"""Small host-side helpers shared by the tests (no method arithmetic of the library)."""
import numpy as np

TIER_SHIFT = 30


def entry(tier: int, owner: int = 0) -> int:
    return (tier << TIER_SHIFT) | owner


def random_jagged(rng, T, B, E, max_len, zero_frac=0.2):
    """Random jagged batch with some empty segments; ids uniform in [0, E)."""
    lengths = rng.integers(0, max_len + 1, size=T * B)
    lengths[rng.random(T * B) < zero_frac] = 0
    offsets = np.zeros(T * B + 1, dtype=np.int64)
    np.cumsum(lengths, out=offsets[1:])
    n = int(offsets[-1])
    ids = rng.integers(0, E, size=n).astype(np.int64)
    row_base = (np.arange(T + 1) * E).astype(np.int64)
    return ids, offsets, row_base, n


def random_placement(rng, R, U, W, p=(0.2, 0.3, 0.5)):
    tier = rng.choice(3, size=R, p=p).astype(np.uint32)
    owner = np.where(tier == 2, rng.integers(0, U, size=R),
                     np.where(tier == 1, rng.integers(0, W, size=R), rng.integers(0, 1 << 20, size=R)))
    return ((tier << TIER_SHIFT) | owner.astype(np.uint32)).astype(np.uint32)


def table_of(offsets, B):
    """Table index of every lookup, from the segment structure."""
    S = len(offsets) - 1
    seg = np.repeat(np.arange(S), np.diff(offsets))
    return seg // B


def dest_numpy(g, placement, U, W, self_):
    """Destination bucket per lookup, vectorised (valid placements only)."""
    e = placement[g]
    tier = e >> TIER_SHIFT
    own = (e & 0x3FFFFFFF).astype(np.int64)
    return np.where(tier == 0, self_, np.where(tier == 1, (self_ // W) * W + own, own)), tier


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    b = x.astype(np.float32).view(np.uint32).astype(np.uint64)
    rounded = b + 0x7FFF + ((b >> 16) & 1)
    return (rounded >> 16).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)
