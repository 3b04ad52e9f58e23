"""Glue used by the tests, the benchmark and the smoke check: turns a
synthetic workload into calls of the C ABI (through the binding in tkv.py).
It plans on the host with the library's own planners, moves plans and inputs
to the GPU with torch, and launches the library's kernels; it computes
nothing itself."""
from __future__ import annotations

import math

import numpy as np
import torch

from . import tkv

PAGE = tkv.PAGE_TOKENS


def bf16_tensor(bits_u16: np.ndarray, device) -> torch.Tensor:
    """numpy uint16 bit patterns -> torch bf16 tensor on `device` (same bits)."""
    t = torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16))
    return t.to(device).view(torch.bfloat16)


def device_kv(n_tokens: int, n_kv_heads: int, seed: int, device, outlier_channels: int = 4, outlier_scale: float = 20.0,
              chunk_tokens: int = 1 << 17):
    """Seeded synthetic K, V bf16 [T, Hkv, 128] generated on the device (input generation only, for runs that are
    timed but not compared with the oracle): N(0,1), `outlier_channels` channels per kv head (seeded choice, fixed
    across tokens) scaled by `outlier_scale`, as workloads.make_kv does on the host."""
    rng = np.random.default_rng(np.random.SeedSequence([seed, 31337]))
    mult = np.ones((n_kv_heads, tkv.HEAD_DIM), np.float32)
    for h in range(n_kv_heads):
        mult[h, rng.choice(tkv.HEAD_DIM, outlier_channels, replace=False)] = outlier_scale
    mult = torch.from_numpy(mult).to(device)
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFF)
    out = []
    for _ in range(2):
        t = torch.empty((n_tokens, n_kv_heads, tkv.HEAD_DIM), dtype=torch.bfloat16, device=device)
        for a in range(0, n_tokens, chunk_tokens):
            b = min(n_tokens, a + chunk_tokens)
            x = torch.randn((b - a, n_kv_heads, tkv.HEAD_DIM), dtype=torch.float32, device=device, generator=g)
            t[a:b] = (x * mult).to(torch.bfloat16)
        out.append(t)
    return out[0], out[1]


def device_q(batch: int, n_q_heads: int, seed: int, device):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 7919 + 13) & 0x7FFFFFFF)
    return torch.randn((batch, n_q_heads, tkv.HEAD_DIM), dtype=torch.float32, device=device, generator=g).to(torch.bfloat16)


class PagedCache:
    """Pool + page tables of one layer for a batch of sequences."""

    def __init__(self, n_kv_heads: int, seq_bits: list, device, pool_factor: float = 1.0, shuffle_seed: int = 1,
                 fill: int | None = None, key_axis: int = tkv.TKV_KEYS_PER_TOKEN, alloc_pool: bool = True):
        self.device = torch.device(device)
        self.n_kv_heads = n_kv_heads
        self.seq_bits = [np.ascontiguousarray(b, np.uint8) for b in seq_bits]
        if key_axis == tkv.TKV_KEYS_PER_CHANNEL:
            # INT2 keys per channel need whole blocks of 32 tokens: the library moves the rest to INT4
            self.seq_bits = [tkv.tkv_route_residual(b) for b in self.seq_bits]
        need2 = sum(math.ceil(int((b == 2).sum()) / PAGE) for b in self.seq_bits)
        need4 = sum(math.ceil(int((b == 4).sum()) / PAGE) for b in self.seq_bits)
        self.P2 = max(1, int(math.ceil(need2 * pool_factor)))
        self.P4 = max(1, int(math.ceil(need4 * pool_factor)))
        self.desc = tkv.tkv_desc.make(n_kv_heads, self.P2, self.P4, int2_key_axis=key_axis)
        self.alloc = tkv.tkv_alloc_create(self.desc, shuffle_seed)
        self.seqs = [tkv.tkv_seq_create() for _ in self.seq_bits]
        nbytes = tkv.tkv_pool_bytes(self.desc)
        self.pool_bytes = nbytes
        if not alloc_pool:
            self.pool = None      # the caller passes a pool to every call (one pool per layer)
        elif fill is None:
            self.pool = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        else:
            self.pool = torch.full((nbytes,), fill, dtype=torch.uint8, device=self.device)
        self.bit_map = torch.zeros(self.P2 + self.P4, dtype=torch.uint8, device=self.device)
        self.status = torch.zeros(1, dtype=torch.int32, device=self.device)
        # host plan of the whole append (Q1)
        slots, wps, wss = [], [], []
        base = 0
        for s, b in zip(self.seqs, self.seq_bits):
            sl, wp, ws = tkv.tkv_plan_append(self.alloc, s, b, base)
            slots.append(sl); wps.append(wp); wss.append(ws)
            base += b.size
        self.n_tokens = base
        self.slot_ids = np.concatenate(slots) if slots else np.zeros(0, np.int32)
        self.work_pages = np.concatenate(wps) if wps else np.zeros(0, np.int32)
        self.work_src = np.concatenate(wss) if wss else np.zeros((0, PAGE), np.int32)
        self.tag_bits = np.concatenate(self.seq_bits) if self.seq_bits else np.zeros(0, np.uint8)
        # page table (INT2 pages first per sequence)
        ids = [tkv.tkv_seq_page_ids(s) for s in self.seqs]
        self.page_indptr = np.concatenate([[0], np.cumsum([i.size for i in ids])]).astype(np.int32)
        self.page_ids = np.concatenate(ids).astype(np.int32) if ids else np.zeros(0, np.int32)
        self.n_tok2 = np.array([tkv.tkv_seq_n_tokens(s, 2) for s in self.seqs], np.int32)
        self.n_tok4 = np.array([tkv.tkv_seq_n_tokens(s, 4) for s in self.seqs], np.int32)
        d = self.device
        self.d_work_pages = torch.from_numpy(self.work_pages).to(d)
        self.d_work_src = torch.from_numpy(self.work_src).to(d)
        self.d_tag_bits = torch.from_numpy(self.tag_bits).to(d)
        self.d_page_indptr = torch.from_numpy(self.page_indptr).to(d)
        self.d_page_ids = torch.from_numpy(self.page_ids).to(d)
        self.d_n_tok2 = torch.from_numpy(self.n_tok2).to(d)
        self.d_n_tok4 = torch.from_numpy(self.n_tok4).to(d)
        self._plan = None

    def close(self):
        for s in self.seqs:
            tkv.tkv_seq_destroy(s)
        tkv.tkv_alloc_destroy(self.alloc)
        self.seqs, self.alloc = [], None

    # -- Q2-Q5
    def append(self, K: torch.Tensor, V: torch.Tensor, pool=None, stream=None, prepare=False):
        """prepare=True returns the call with its arguments marshalled once (tkv.Prepared) instead of making it."""
        return tkv.tkv_quantize_append(self.desc, self.pool if pool is None else pool, self.bit_map, K, V,
                                       self.d_tag_bits, self.d_work_pages, self.d_work_src, self.status, stream,
                                       prepare=prepare)

    # -- P1
    def gather(self, K_out: torch.Tensor, V_out: torch.Tensor, pool=None, stream=None):
        """Prefill gather of every cached token back into its original row (fp16 [T,Hkv,D])."""
        tkv.tkv_gather_dequant(self.desc, self.pool if pool is None else pool, self.bit_map, self.d_work_pages,
                               self.d_work_src, K_out, V_out, self.status, stream)

    # -- D1
    def plan_decode(self, target_items: int):
        items, sip = tkv.tkv_plan_decode(self.desc, self.page_indptr, self.n_tok2, self.n_tok4, target_items)
        self._plan = (torch.from_numpy(items).to(self.device), torch.from_numpy(sip).to(self.device), items, sip)
        return items, sip

    # -- D2-D7
    def decode(self, q: torch.Tensor, out: torch.Tensor | None = None, workspace=None, pool=None, stream=None,
               prepare=False):
        """prepare=True returns the call (tkv.Prepared) instead of `out`; `out` and `workspace` must then be given."""
        assert self._plan is not None, "call plan_decode first"
        assert not prepare or (out is not None and workspace is not None)
        d_items, d_sip, items, _ = self._plan
        B, Hq = int(q.shape[0]), int(q.shape[1])
        if out is None:
            out = torch.empty((B, Hq, tkv.HEAD_DIM), dtype=torch.float32, device=self.device)
        if workspace is None:
            workspace = self.workspace(Hq)
        sm_scale = np.float32(1.0 / math.sqrt(tkv.HEAD_DIM))
        call = tkv.tkv_decode_attention(self.desc, self.pool if pool is None else pool, self.bit_map, q,
                                        self.d_page_indptr, self.d_page_ids, self.d_n_tok2, self.d_n_tok4, d_items, d_sip,
                                        float(sm_scale), out, workspace, self.status, stream, prepare=prepare)
        return call if prepare else out

    def decode_static(self, q: torch.Tensor, out: torch.Tensor, pool=None, stream=None):
        """D2-D7 with the partials in the library's fixed device array: nothing is allocated here either
        (`out` comes from the caller)."""
        d_items, d_sip, _, _ = self._plan
        sm_scale = np.float32(1.0 / math.sqrt(tkv.HEAD_DIM))
        tkv.tkv_decode_attention_static(self.desc, self.pool if pool is None else pool, self.bit_map, q,
                                        self.d_page_indptr, self.d_page_ids, self.d_n_tok2, self.d_n_tok4, d_items,
                                        d_sip, float(sm_scale), out, self.status, stream)
        return out

    def decode_split(self, q: torch.Tensor, workspace, pool=None, stream=None, prepare=False):
        """D2-D6 only (used by the benchmark to time the split kernel by itself)."""
        d_items = self._plan[0]
        sm_scale = np.float32(1.0 / math.sqrt(tkv.HEAD_DIM))
        return tkv.tkv_decode_split(self.desc, self.pool if pool is None else pool, self.bit_map, q, self.d_page_indptr,
                                    self.d_page_ids, self.d_n_tok2, self.d_n_tok4, d_items, float(sm_scale), workspace,
                                    self.status, stream, prepare=prepare)

    def workspace(self, n_q_heads: int) -> torch.Tensor:
        n_items = self._plan[2].shape[0]
        nbytes = max(16, tkv.tkv_decode_workspace_bytes(self.desc, n_items, n_q_heads))
        return torch.empty(nbytes, dtype=torch.uint8, device=self.device)

    def kv_bytes(self) -> int:
        """Algorithmic bytes a decode step reads from the pool (96 B per INT2
        token, 160 B per INT4 token, per kv head)."""
        return int(self.n_kv_heads * (96 * int(self.n_tok2.sum()) + 160 * int(self.n_tok4.sum())))


def default_target_items(n_kv_heads: int, device=None) -> int:
    """Work items over the batch: one wavefront serves one (item, kv head), and
    the decode kernel's register footprint lets three wavefronts share a SIMD,
    so 12 per compute unit fill the device in a single round."""
    props = torch.cuda.get_device_properties(device if device is not None else torch.cuda.current_device())
    waves = props.multi_processor_count * 4 * 3
    return max(1, waves // n_kv_heads)
