"""Seeded synthetic inputs for the decode / append hot path.

This module only GENERATES inputs: token traces with triaxial tags, the
per-token bitwidth arrays derived from them, and random bf16 q / K / V.  It
holds none of the quantiser's or the attention kernel's arithmetic and is
imported by the tests, the benchmark and the smoke check alike; both the HIP
path and the CPU oracle are fed from the arrays it returns.

The traces stand in for the paper's agentic workloads (multi-turn function
calling and computer-use trajectories, Sec. 4.1), which are not available
here: only their SHAPE is reproduced -- long multi-turn contexts, screenshot
observations as 1024-token image blocks, 65-75 % of prefill tokens at INT2
(Appendix B, Table 6), the most recent turn and the instruction prefix kept
at INT4.  Tag space: temporal x modal x semantic (Sec. 3.1, Table 1).

bf16 / fp16 tensors are numpy uint16 arrays of bit patterns.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

TEMPORAL = ("older", "turn_m2", "turn_m1", "current")
MODAL = ("text", "image")
SEMANTIC = ("inst", "user", "assistant", "reasoning", "tool_call", "obs", "delim")
N_TAGS = len(TEMPORAL) * len(MODAL) * len(SEMANTIC)  # 56

PAGE_TOKENS = 64
HEAD_DIM = 128
GROUP = 32


def tag_code(temporal: int, modal: int, semantic: int) -> int:
    return (temporal * len(MODAL) + modal) * len(SEMANTIC) + semantic


def tag_fields(code):
    code = np.asarray(code)
    return code // 14, (code // 7) % 2, code % 7


# --------------------------------------------------------------------- bf16
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def normal_bf16(rng: np.random.Generator, shape, chunk: int = 1 << 24) -> np.ndarray:
    """N(0,1) samples rounded to bf16, generated in chunks to bound memory."""
    n = int(np.prod(shape))
    out = np.empty(n, np.uint16)
    for s in range(0, n, chunk):
        e = min(n, s + chunk)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


def make_kv(seed_seq: np.random.SeedSequence, n_tokens: int, n_kv_heads: int,
            outlier_channels: int = 4, outlier_scale: float = 20.0, chunk_tokens: int = 8192):
    """K, V bf16 bits [T, Hkv, D] ~ N(0,1); per kv head, `outlier_channels`
    seeded channel indices (fixed across tokens) are scaled by `outlier_scale`
    in both K and V (key-channel outliers are the paper's stated motive for
    its INT2 key treatment, Sec. 3.2.1).  Tokens are generated in chunks, each
    from its own spawned seed, so the result does not depend on the number of
    worker threads.  Returns (K, V, outlier_idx[Hkv, n])."""
    from concurrent.futures import ThreadPoolExecutor
    s_k, s_v, s_o = seed_seq.spawn(3)
    rng_o = np.random.default_rng(s_o)
    idx = np.stack([rng_o.choice(HEAD_DIM, outlier_channels, replace=False) for _ in range(n_kv_heads)]) \
        if outlier_channels else np.zeros((n_kv_heads, 0), np.int64)
    mult = np.ones((n_kv_heads, HEAD_DIM), np.float32)
    for h in range(n_kv_heads):
        mult[h, idx[h]] = outlier_scale
    n_chunks = max(1, -(-n_tokens // chunk_tokens))
    out = []
    for s in (s_k, s_v):
        buf = np.empty((n_tokens, n_kv_heads, HEAD_DIM), np.uint16)
        seeds = s.spawn(n_chunks)

        def fill(i):
            t0, t1 = i * chunk_tokens, min(n_tokens, (i + 1) * chunk_tokens)
            x = np.random.default_rng(seeds[i]).standard_normal((t1 - t0, n_kv_heads, HEAD_DIM), dtype=np.float32)
            x *= mult
            buf[t0:t1] = f32_to_bf16_bits(x)

        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(n_chunks)))
        out.append(buf)
    return out[0], out[1], idx


def make_q(seed_seq: np.random.SeedSequence, batch: int, n_q_heads: int) -> np.ndarray:
    """q bf16 bits [B, Hq, D] ~ N(0,1) (no outlier scaling: scaling q as well
    drives the softmax to one-hot, a degenerate test)."""
    return normal_bf16(np.random.default_rng(seed_seq), (batch, n_q_heads, HEAD_DIM))


# --------------------------------------------------------------------- traces
def segment_trace(rng: np.random.Generator, n_tokens: int, n_segments: int = 8):
    """`n_segments` equal contiguous segments with random tags; half of the
    segments (seeded choice) are INT4, half INT2.  Returns (tags i16, bits u8)."""
    seg = n_tokens // n_segments
    tags = np.empty(n_tokens, np.int16)
    bits = np.empty(n_tokens, np.uint8)
    int4 = np.zeros(n_segments, bool)
    int4[rng.choice(n_segments, n_segments // 2, replace=False)] = True
    for s in range(n_segments):
        a, b = s * seg, (n_tokens if s == n_segments - 1 else (s + 1) * seg)
        tags[a:b] = tag_code(int(rng.integers(4)), 0, int(rng.integers(7)))
        bits[a:b] = 4 if int4[s] else 2
    return tags, bits


def agentic_trace(rng: np.random.Generator, ctx: int, image_share: float,
                  median_len: float = 400.0, sigma: float = 1.0, recent: int = 512,
                  image_block: int = 1024) -> np.ndarray:
    """Tag codes i16 [ctx] of one synthetic agent trajectory: an instruction
    prefix, then turns (user -> {reasoning, tool_call, obs}* -> assistant),
    text segment lengths lognormal(median, sigma) clipped to [16, 4096],
    observations turned into `image_block`-token image blocks until about
    `image_share` of the tokens are image tokens.  Temporal tags count turns
    back from the last one; the last `recent` tokens are `current`."""
    sem = {n: i for i, n in enumerate(SEMANTIC)}
    seg_sem, seg_mod, seg_len, seg_turn = [], [], [], []
    total, turn, img = 0, 0, 0

    def text_len():
        return int(np.clip(round(float(rng.lognormal(np.log(median_len), sigma))), 16, 4096))

    def push(s, m, n, t):
        nonlocal total, img
        n = min(n, ctx - total)
        if n <= 0:
            return
        seg_sem.append(s); seg_mod.append(m); seg_len.append(n); seg_turn.append(t)
        total += n
        img += n if m else 0

    push(sem["inst"], 0, text_len(), 0)
    while total < ctx:
        turn += 1
        push(sem["delim"], 0, 4, turn)
        push(sem["user"], 0, text_len(), turn)
        for _ in range(int(rng.integers(1, 5))):
            if total >= ctx:
                break
            push(sem["reasoning"], 0, text_len(), turn)
            push(sem["tool_call"], 0, max(16, text_len() // 4), turn)
            want_img = image_share > 0 and (img < image_share * (total + image_block))
            if want_img:
                push(sem["obs"], 1, image_block, turn)
            else:
                push(sem["obs"], 0, text_len(), turn)
        push(sem["assistant"], 0, text_len(), turn)
    last_turn = seg_turn[-1]
    tags = np.empty(ctx, np.int16)
    pos = 0
    for s, m, n, t in zip(seg_sem, seg_mod, seg_len, seg_turn):
        back = last_turn - t
        temporal = 3 if back == 0 else (2 if back == 1 else (1 if back == 2 else 0))
        if s == sem["inst"]:
            temporal = 0
        tags[pos:pos + n] = tag_code(temporal, m, s)
        pos += n
    # the most recent `recent` tokens count as the current turn
    tmp, mod, se = tag_fields(tags[ctx - recent:])
    tags[ctx - recent:] = (3 * 2 + mod) * 7 + se
    return tags


def bits_table(tag_counts: np.ndarray, rng: np.random.Generator, f4_target: float) -> np.ndarray:
    """Tag -> bitwidth table of a synthetic workload: an INPUT recipe, not the allocator under test (no
    calibration data exists here, so there are no distortions to allocate by).  Tags get a seeded random
    priority and are set to 4 bits in priority order while their tokens still fit an INT4 token share of
    f4_target; `current` and `inst` tags come first and image tags never, as the paper's allocations keep
    recent and instruction tokens at INT4 and route screenshots to INT2 (Appendix B)."""
    n = tag_counts.astype(np.float64)
    temporal, modal, semantic = tag_fields(np.arange(N_TAGS))
    gain = rng.lognormal(0.0, 1.0, N_TAGS)
    gain[modal == 1] = 0.0
    gain[semantic == 0] = 1e6
    gain[temporal == 3] = 1e9
    table = np.full(N_TAGS, 2, np.uint8)
    budget = 2.0 * f4_target * n.sum()  # extra bits available beyond all-INT2
    for k in np.argsort(-gain, kind="stable"):
        if n[k] == 0 or gain[k] == 0.0:
            continue
        if 2.0 * n[k] <= budget:
            table[k] = 4
            budget -= 2.0 * n[k]
    return table


# --------------------------------------------------------------------- workloads
@dataclass
class Workload:
    """One synthetic decode / append workload (arrays are host numpy)."""
    name: str
    n_q_heads: int
    n_kv_heads: int
    seq_lens: np.ndarray            # i64 [B]
    bits: list                      # per sequence: u8 [len]
    tags: list                      # per sequence: i16 [len]
    seed: int
    n_layers: int = 1
    notes: str = ""
    streams: list = field(default_factory=list)

    @property
    def batch(self) -> int:
        return len(self.seq_lens)

    @property
    def n_tokens(self) -> int:
        return int(np.sum(self.seq_lens))

    @property
    def seq_indptr(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_lens)]).astype(np.int64)

    def all_bits(self) -> np.ndarray:
        return np.concatenate(self.bits) if self.bits else np.zeros(0, np.uint8)

    def f4(self) -> float:
        b = self.all_bits()
        return float(np.mean(b == 4)) if b.size else 0.0

    def kv_bytes_per_layer(self) -> int:
        """Algorithmic packed bytes one decode step reads: 96 B per INT2
        token and 160 B per INT4 token per kv head (codes + fp16 scale and
        zero of K and V)."""
        b = self.all_bits()
        return int(self.n_kv_heads * (96 * np.sum(b == 2) + 160 * np.sum(b == 4)))

    def seeds(self, layer: int = 0):
        """(kv, q) SeedSequences of one layer (independent per layer)."""
        ss = np.random.SeedSequence([self.seed, 7919, layer])
        return ss.spawn(2)

    def make_inputs(self, layer: int = 0):
        s_kv, s_q = self.seeds(layer)
        K, V, oidx = make_kv(s_kv, self.n_tokens, self.n_kv_heads)
        q = make_q(s_q, self.batch, self.n_q_heads)
        return q, K, V, oidx


def _agentic(name, seed, batch, ctx_list, Hq, Hkv, image_share, f4, n_layers=1, notes=""):
    ss = np.random.SeedSequence([seed, 104729])
    s_tr, s_tab = ss.spawn(2)
    rngs = [np.random.default_rng(s) for s in s_tr.spawn(batch)]
    tags = [agentic_trace(r, int(c), image_share) for r, c in zip(rngs, ctx_list)]
    counts = np.bincount(np.concatenate(tags), minlength=N_TAGS)
    table = bits_table(counts, np.random.default_rng(s_tab), f4)
    bits = [table[t] for t in tags]
    return Workload(name, Hq, Hkv, np.asarray(ctx_list, np.int64), bits, tags, seed, n_layers, notes)


def config(name: str, scale: float = 1.0) -> Workload:
    """The five benchmark configurations.  `scale` < 1 shrinks context lengths
    (and the append size) for fast tests while keeping every other property.

    cfg1  small single decode step: B=1, Hq=4, Hkv=1, ctx 2048, 8 segments, seed 0
    cfg2  Qwen3-VL-32B-shaped layer: B=8, Hq=64, Hkv=8, ctx 32768, agentic traces, seed 1
    cfg3  ~100K-token computer-use step: B=4, Hq=4, Hkv=1, ctx 102400, 40 % image, seed 2
    cfg4  append of 65536 new tokens, Hkv=8, 8 segments, seed 3
    cfg5  Llama-3-70B-shaped step: 80 layers, B=32, Hq=64, Hkv=8, ctx lognormal 4K..128K, seed 4
    """
    def sc(n, lo=PAGE_TOKENS):
        return max(lo, int(round(n * scale)))

    if name == "cfg1":
        rng = np.random.default_rng(np.random.SeedSequence([0, 1299709]))
        tags, bits = segment_trace(rng, sc(2048, 8 * 8), 8)
        return Workload("cfg1", 4, 1, np.asarray([tags.size]), [bits], [tags], 0)
    if name == "cfg2":
        return _agentic("cfg2", 1, 8, [sc(32768, 640)] * 8, 64, 8, 0.25, 0.30)
    if name == "cfg3":
        return _agentic("cfg3", 2, 4, [sc(102400, 640)] * 4, 4, 1, 0.40, 0.25,
                        notes="pool sized for 16 sequences, pages scattered")
    if name == "cfg4":
        rng = np.random.default_rng(np.random.SeedSequence([3, 1299709]))
        tags, bits = segment_trace(rng, sc(65536, 8 * 8), 8)
        return Workload("cfg4", 8, 8, np.asarray([tags.size]), [bits], [tags], 3)
    if name == "cfg5":
        rng = np.random.default_rng(np.random.SeedSequence([4, 15485863]))
        ctx = np.clip(np.round(rng.lognormal(np.log(24576.0), 0.8, 32)), 4096, 131072)
        ctx = np.maximum(640, np.round(ctx * scale)).astype(np.int64)
        return _agentic("cfg5", 4, 32, list(ctx), 64, 8, 0.10, 0.30, n_layers=80)
    raise KeyError(name)
