"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds only random draws, shape tables and dtype plumbing (bf16 rounding of the
drawn values); none of the method's arithmetic lives here.  Values stand in for
the served prompts and released model weights of the paper's evaluation
(Section 6), which fix only shapes: decoder dimensions of the Llama-3 family,
prompt lengths from hundreds to a few thousand tokens.
"""
import numpy as np

# name -> (hidden, n_q_heads, n_kv_heads, head_dim, ffn, rms_eps, rope_base)
SHAPES = {
    "tiny":     (16, 4, 2, 8, 24, 1e-6, 10000.0),
    "config1":  (256, 4, 4, 64, 1024, 1e-6, 10000.0),
    "medium":   (512, 8, 2, 128, 1536, 1e-5, 500000.0),
    "medium64": (384, 6, 3, 64, 1024, 1e-5, 10000.0),
    "llama8b":  (4096, 32, 8, 128, 14336, 1e-5, 500000.0),
    "llama70b": (8192, 64, 8, 128, 28672, 1e-5, 500000.0),
    "phi4":     (5120, 40, 10, 128, 17920, 1e-5, 250000.0),   # the third model of the paper's evaluation (Section 6)
}
# a test shape whose fused q/k/v weight gradient has 48 x 8 = 384 output tiles in three row ranges
SHAPES["wideqkv"] = (2048, 64, 16, 128, 512, 1e-5, 10000.0)
# widths that are multiples of neither 8 nor 16 elements: every kernel takes its element-wise path
SHAPES["odd"] = (20, 2, 1, 12, 22, 1e-5, 10000.0)
SHAPE_FIELDS = ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "rms_eps", "rope_base")


def shape_dict(name):
    return dict(zip(SHAPE_FIELDS, SHAPES[name]))


def f32_to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def quantize(x, dtype):
    """Round an fp32 array to the storage dtype ("f32" or "bf16"); returns fp32 values."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return bf16_bits_to_f32(f32_to_bf16_bits(x))
    return x


def normal(rng, shape, std, dtype):
    return quantize(rng.standard_normal(shape, dtype=np.float32) * np.float32(std), dtype)


def uniform_cu(n_seqs, seqlen):
    return np.arange(n_seqs + 1, dtype=np.int32) * np.int32(seqlen)


def ragged_cu(lengths):
    cu = np.zeros(len(lengths) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(lengths, dtype=np.int64))
    return cu


def random_lengths(n_seqs, lo, hi, seed):
    """Prompt lengths uniform in [lo, hi] (inclusive)."""
    rng = np.random.default_rng(seed)
    return rng.integers(lo, hi + 1, size=n_seqs).astype(np.int64)


def keep_mask(T, p, seed):
    rng = np.random.default_rng(seed)
    return (rng.random(T) < p).astype(np.uint8)


def layer_weights(shape, seed, dtype, std=0.02, gain_std=0.0):
    """W ~ N(0, std) for the seven matrices; norm gains 1 (+ N(0, gain_std))."""
    rng = np.random.default_rng(seed)
    H, Hq, Hkv, D, F = (shape[k] for k in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn"))
    W = {
        "Wq": normal(rng, (Hq * D, H), std, dtype),
        "Wk": normal(rng, (Hkv * D, H), std, dtype),
        "Wv": normal(rng, (Hkv * D, H), std, dtype),
        "Wo": normal(rng, (H, Hq * D), std, dtype),
        "Wg": normal(rng, (F, H), std, dtype),
        "Wu": normal(rng, (F, H), std, dtype),
        "Wd": normal(rng, (H, F), std, dtype),
    }
    for k in ("g1", "g2"):
        W[k] = quantize(1.0 + rng.standard_normal(H, dtype=np.float32) * np.float32(gain_std), dtype)
    return W


def drawn_record(shape, T, seed, dtype, std=1.0):
    """Record tensors drawn independently ~ N(0, std) (all but LSE, which the
    caller derives from the drawn Q and K)."""
    rng = np.random.default_rng(seed)
    H, Hq, Hkv, D, F = (shape[k] for k in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn"))
    widths = dict(X=H, X2=H, Q=Hq * D, K=Hkv * D, V=Hkv * D, O=Hq * D, G=F, U=F)
    return {k: normal(rng, (T, w), std, dtype) for k, w in widths.items()}


def activations(T, width, seed, dtype, std=1.0):
    return normal(np.random.default_rng(seed), (T, width), std, dtype)


PROJECTIONS = ("q", "k", "v", "o", "g", "u", "d")


def lora_adapters(shape, rank, seed, dtype, projections=PROJECTIONS, std=0.05):
    """Adapter pairs (A [rank, in], B [out, rank]) ~ N(0, std) for the named projections.
    (The usual initialisation B = 0 makes half of the gradients trivially zero, so both are drawn.)"""
    rng = np.random.default_rng(seed)
    H, Hq, Hkv, D, F = (shape[k] for k in ("hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn"))
    dims = dict(q=(Hq * D, H), k=(Hkv * D, H), v=(Hkv * D, H), o=(H, Hq * D), g=(F, H), u=(F, H), d=(H, F))
    out = {}
    for p in PROJECTIONS:  # fixed draw order whatever subset is asked for
        o, i = dims[p]
        A, B = normal(rng, (rank, i), std, dtype), normal(rng, (o, rank), std, dtype)
        if p in projections:
            out[p] = (A, B)
    return out


def preference_batch(prompt_lens, response_lens, vocab, seed):
    """Layout of a preference-alignment batch (Section 4.1, Section 6 of the paper: prompts answered by a
    chosen and a rejected response): all prompts first, then for prompt g its responses in order.
    response_lens[g] = lengths of the responses of prompt g (two for a pair: chosen, rejected).
    Returns dict: cu [n_seqs+1], prefix [n_seqs] (-1 for prompts, the prompt's index for responses),
    positions [T] (index in the sequence plus the prefix length), tokens [T] (random ids), and the scored
    items sorted by row: item_row, item_label, item_slot (slot = running index of the response).  Token 0 of
    a response is scored from the last row of its prompt, token i+1 from row i of the response."""
    rng = np.random.default_rng(seed)
    n_p = len(prompt_lens)
    lens = [int(n) for n in prompt_lens] + [int(n) for rl in response_lens for n in rl]
    cu = ragged_cu(lens)
    T = int(cu[-1])
    prefix = np.full(len(lens), -1, dtype=np.int32)
    positions = np.zeros(T, dtype=np.int32)
    for s in range(n_p):
        positions[cu[s]:cu[s + 1]] = np.arange(lens[s])
    tokens = rng.integers(0, vocab, T).astype(np.int32)
    items = []
    s = n_p
    for g, rl in enumerate(response_lens):
        for n in rl:
            prefix[s] = g
            a = int(cu[s])
            positions[a:a + int(n)] = lens[g] + np.arange(int(n))
            slot = s - n_p
            if n > 0 and lens[g] > 0:
                items.append((int(cu[g + 1]) - 1, int(tokens[a]), slot))
            for i in range(int(n) - 1):
                items.append((a + i, int(tokens[a + i + 1]), slot))
            s += 1
    items.sort(key=lambda it: (it[0], it[2]))
    arr = np.asarray(items, dtype=np.int32).reshape(-1, 3)
    return dict(cu=cu, prefix=prefix, positions=positions, tokens=tokens, n_prompts=n_p,
                item_row=arr[:, 0].copy(), item_label=arr[:, 1].copy(), item_slot=arr[:, 2].copy())
