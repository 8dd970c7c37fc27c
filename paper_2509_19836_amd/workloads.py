"""Seeded synthetic inputs and the benchmark's workload table.

This module holds no attention arithmetic: it only draws random tensors,
rounds them to bfloat16 and describes the shapes of the workloads.  It is the
one module both the HIP-path tests and the CPU oracle tests import, so that
both sides see byte-identical inputs.

Tensors are [batch, seq, heads, head_dim].  Host tensors are numpy arrays of
bfloat16 BIT PATTERNS (dtype uint16) plus helpers to widen them exactly.
"""
from dataclasses import dataclass
import numpy as np

BASE_SEED = 250919836


def f32_to_bf16_bits(x):
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (uint16)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    rounded = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(bits):
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(bits):
    """Exact widening of bfloat16 bit patterns to float64."""
    return bf16_bits_to_f32(bits).astype(np.float64)


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    q_heads: int
    kv_heads: int
    head_dim: int
    shard_tokens: int     # rows of the local Q chunk = rows of one KV chunk
    shards: int           # G, number of simulated devices on the ring
    mask: str             # "full", "causal" (contiguous split) or "zigzag"
    head_scale: bool = False   # per-(tensor, batch, head) factor ~ U(0.5, 2)

    @property
    def seq(self):
        return self.shard_tokens * self.shards

    @property
    def scale(self):
        return 1.0 / float(np.sqrt(self.head_dim))


# The five configurations of the benchmark definition, index = config number.
WORKLOADS = {
    1: Workload("tiny_ring_1k", 1, 2, 2, 64, 256, 4, "causal"),
    2: Workload("llama7b_zigzag_128k", 1, 32, 32, 128, 16384, 8, "zigzag"),
    3: Workload("gqa_zigzag_256k", 1, 64, 8, 128, 32768, 8, "zigzag"),
    4: Workload("full_lmm_256k", 2, 32, 32, 128, 65536, 4, "full", True),
    5: Workload("zigzag_1m", 1, 32, 32, 128, 131072, 8, "zigzag"),
}


def scaled_down(w, shard_tokens, batch=None, q_heads=None, kv_heads=None):
    """Same structure (mask, grouping, head_dim, value distribution) at a
    size the fp64 oracle can do exhaustively."""
    return Workload(w.name + f"_s{shard_tokens}", batch or w.batch, q_heads or w.q_heads,
                    kv_heads or w.kv_heads, w.head_dim, shard_tokens, w.shards, w.mask,
                    w.head_scale)


def _draw(seed, shape, head_scale):
    rng = np.random.Generator(np.random.PCG64(seed))
    x = rng.standard_normal(shape, dtype=np.float32)
    if head_scale:
        B, _, H, _ = shape
        s = rng.uniform(0.5, 2.0, size=(B, 1, H, 1)).astype(np.float32)
        x = x * s
    return x


def host_tensors(w, cfg_index=0, seed_offset=0):
    """Whole-sequence Q, K, V, dO as (float32 draws, bf16 bit patterns).

    Returns a dict name -> (f32 array, uint16 array), each
    [batch, seq, heads, head_dim] in GLOBAL token order.  Seeds: base + 100 *
    config index, +0 Q, +1 K, +2 V, +3 dO."""
    base = BASE_SEED + 100 * cfg_index + 1000 * seed_offset
    out = {}
    shapes = {
        "q": (w.batch, w.seq, w.q_heads, w.head_dim),
        "k": (w.batch, w.seq, w.kv_heads, w.head_dim),
        "v": (w.batch, w.seq, w.kv_heads, w.head_dim),
        "do": (w.batch, w.seq, w.q_heads, w.head_dim),
    }
    for n, (name, shape) in enumerate(shapes.items()):
        x = _draw(base + n, shape, w.head_scale and name != "do")
        out[name] = (x, f32_to_bf16_bits(x))
    return out


def block_sparse_pattern(n_blocks, density, seed):
    """Seeded block-sparse attention pattern over global token blocks: an n_blocks x n_blocks uint8
    matrix (row: query block, column: key block) whose entries are open with probability `density`,
    with the diagonal always open so that every token keeps at least itself."""
    rng = np.random.Generator(np.random.PCG64(seed))
    pat = (rng.random((n_blocks, n_blocks)) < density).astype(np.uint8)
    np.fill_diagonal(pat, 1)
    return pat


def local_block_mask(pattern, pos_q, pos_k, block_rows, global_block=None):
    """The slice of a global block pattern that a ring step sees, on LOCAL row blocks of block_rows
    rows: entry [a][b] is the pattern entry of the global blocks (of global_block tokens; default
    block_rows) that hold local row blocks a and b.  pos_q / pos_k: global positions of the local rows;
    every local block must lie inside one global block.  That holds for the contiguous and zigzag splits
    when block_rows = global_block divides the piece length, and for the two balanced splits of
    block-wise sparse attention (slice i or stripe i of every block) with block_rows = global_block / G."""
    global_block = global_block or block_rows
    pos_q, pos_k = np.asarray(pos_q), np.asarray(pos_k)
    blocks = []
    for pos in (pos_q, pos_k):
        if pos.size % block_rows:
            raise ValueError("the chunk is not a whole number of local row blocks")
        g = (pos // global_block).reshape(-1, block_rows)
        if not (g == g[:, :1]).all():
            raise ValueError("local row blocks straddle global blocks")
        blocks.append(g[:, 0])
    return np.ascontiguousarray(pattern[np.ix_(blocks[0], blocks[1])])


def lm_head_tensors(seed, n_tokens, d_model, vocab, ignored=0):
    """Seeded inputs of the fused LM head + loss: H_last ~ N(0, 1) and W_head ~ N(0, 4/d) as bfloat16
    bit patterns (logits of standard deviation about 2, the spread of a trained head's logits), targets
    uniform over the vocabulary, the first `ignored` of them set to -100 (tokens without a loss)."""
    rng = np.random.Generator(np.random.PCG64(seed))
    H = f32_to_bf16_bits(rng.standard_normal((n_tokens, d_model), dtype=np.float32))
    W = f32_to_bf16_bits(rng.standard_normal((vocab, d_model), dtype=np.float32) * np.float32(2.0 / np.sqrt(d_model)))
    Y = rng.integers(0, vocab, n_tokens, dtype=np.int64)
    Y[:ignored] = -100
    return H, W, Y
