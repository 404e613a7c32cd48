"""Thin decode-loop driver over the C-ABI calls: owns the device buffers (weight
arena, paged KV cache, per-row state, outputs, workspace) as torch tensors and
chains  hydra_draft_tree -> tree_verify_forward -> accept_greedy -> kv_compact.

No arithmetic of the method happens here; torch is used to allocate memory, to
copy results into a log, and to provide the stream.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Optional, Sequence

import torch

from . import binding as hb


def chain_parent(T: int) -> List[int]:
    return [-1] + list(range(T - 1))


class _Outputs:
    def __init__(self, ctx: hb.Hydra, B: int, d: int, V: int, dev, want_logits: bool):
        T, P = ctx.T, ctx.depth + 1
        i32, f32 = torch.int32, torch.float32
        self.tree_tokens = torch.zeros(B, T, dtype=i32, device=dev)
        self.hidden = torch.zeros(B, T, d, dtype=f32, device=dev)
        self.argmax = torch.zeros(B, T, dtype=i32, device=dev)
        self.margin = torch.zeros(B, T, dtype=f32, device=dev)
        self.logits = torch.zeros(B, T, V, dtype=f32, device=dev) if want_logits else None
        self.n_acc = torch.zeros(B, dtype=i32, device=dev)
        self.path = torch.zeros(B, P, dtype=i32, device=dev)
        self.next_root = torch.zeros(B, dtype=i32, device=dev)
        self.last_node = torch.zeros(B, dtype=i32, device=dev)
        self.kv_index = torch.zeros(B, P, 2, dtype=i32, device=dev)


class Session:
    """`shape` needs attributes d, NL, H, Dh, F, V, dtype ('f32'|'bf16'), K, mlp_layers, rms_eps,
    rope_theta, include_root_embedding.  `get_tensor(name)` returns the named weight as a
    device tensor in the model dtype (names as in the weight generator)."""

    def __init__(self, shape, parent: Sequence[int], B: int, max_len: int,
                 get_tensor: Callable[[str], torch.Tensor], device="cuda:0", prefill_chunk: int = 64,
                 page_perm_seed: Optional[int] = None, want_logits: bool = False, max_pos: Optional[int] = None):
        self.shape, self.B, self.dev = shape, B, torch.device(device)
        self.parent = list(parent)
        self.dtype_code = hb.HYDRA_BF16 if shape.dtype == "bf16" else hb.HYDRA_F32
        self.tdtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.want_logits = want_logits
        self.prefill_chunk = min(prefill_chunk, 128)
        self._max_pos = max_pos or (max_len + 256)
        torch.cuda.set_device(self.dev)
        self._next_slot = 0
        self._ctx: Dict[str, hb.Hydra] = {}
        self._out: Dict[str, _Outputs] = {}
        self.main = self._make_ctx("main", self.parent)
        # weights
        self.arena = torch.empty(self.main.weights_bytes(), dtype=torch.uint8, device=self.dev)
        self._bind(self.main)
        self._load_weights(get_tensor)
        # KV cache
        T_max = max(len(self.parent), self.prefill_chunk)
        self.max_pages = (max_len + T_max + 15) // 16
        self.n_pages = B * self.max_pages
        n_el = shape.NL * self.n_pages * shape.H * 16 * shape.Dh
        cache_dtype = torch.float16 if shape.dtype == "bf16" else torch.float32     # 2 or 4 bytes per element; content is private
        self.k_pages = torch.zeros(n_el, dtype=cache_dtype, device=self.dev)
        self.v_pages = torch.zeros(n_el, dtype=cache_dtype, device=self.dev)
        if page_perm_seed is None:
            perm = torch.arange(self.n_pages, dtype=torch.int32)
        else:
            g = torch.Generator().manual_seed(page_perm_seed)
            perm = torch.randperm(self.n_pages, generator=g).to(torch.int32)
        self.page_table = perm.reshape(B, self.max_pages).contiguous().to(self.dev)
        self.kv = hb.KV(self.k_pages, self.v_pages, self.page_table, self.n_pages, seq_len_hint=0)
        # state
        self.seq_len = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.h_last = torch.zeros(B, shape.d, dtype=torch.float32, device=self.dev)
        self.root = torch.zeros(B, dtype=torch.int32, device=self.dev)
        self.host_len = 0                     # host upper bound on seq_len (hint only)
        # the bound is tightened without stalling: every few steps seq_len is copied to pinned memory and picked
        # up once the copy has landed
        self._len_pinned = torch.zeros(B, dtype=torch.int32).pin_memory()
        self._len_event: Optional[torch.cuda.Event] = None
        self._growth_since_copy = 0
        self._steps_since_copy = 0
        self.ws = torch.empty(max(self.main.workspace_bytes(B), 256), dtype=torch.uint8, device=self.dev)
        # Hydra++ prefix attention: a one-layer context family of its own (weights, cache, length); it shares the
        # page table with the base cache (same slots, its own page storage)
        self.prefix = bool(getattr(shape, "prefix", 0))
        self._pctx: Dict[int, hb.Hydra] = {}
        if self.prefix:
            self._pnext_slot = 0
            first = self._prefix_ctx_new(self.main.depth + 1)
            self.parena = torch.empty(first.weights_bytes(), dtype=torch.uint8, device=self.dev)
            self._prefix_bind(first)
            for nm, kind in (("attn_norm", hb.W_ATTN_NORM), ("wq", hb.W_WQ), ("wk", hb.W_WK), ("wv", hb.W_WV), ("wo", hb.W_WO),
                             ("ffn_norm", hb.W_FFN_NORM), ("w_gate", hb.W_GATE), ("w_up", hb.W_UP), ("w_down", hb.W_DOWN)):
                first.load_tensor(kind, 0, 0, get_tensor(f"prefix.{nm}"))
            first.load_tensor(hb.W_FINAL_NORM, 0, 0, torch.ones(shape.d, dtype=self.tdtype, device=self.dev))   # never used; kept defined
            torch.cuda.synchronize()
            n_el1 = self.n_pages * shape.H * 16 * shape.Dh
            self.pk_pages = torch.zeros(n_el1, dtype=cache_dtype, device=self.dev)
            self.pv_pages = torch.zeros(n_el1, dtype=cache_dtype, device=self.dev)
            self.pkv = hb.KV(self.pk_pages, self.pv_pages, self.page_table, self.n_pages, seq_len_hint=0)
            self.pseq_len = torch.zeros(B, dtype=torch.int32, device=self.dev)

    # ---- contexts -----------------------------------------------------------
    def _make_ctx(self, name: str, parent: Sequence[int]) -> hb.Hydra:
        s = self.shape
        ctx = hb.Hydra(d=s.d, n_layers=s.NL, n_heads=s.H, head_dim=s.Dh, ffn=s.F, vocab=s.V, dtype=self.dtype_code,
                       rms_eps=s.rms_eps, rope_theta=s.rope_theta, max_pos=self._max_pos, n_draft_heads=s.K,
                       mlp_layers=s.mlp_layers, include_root_embedding=s.include_root_embedding, medusa=getattr(s, "medusa", 0),
                       parent=parent, max_batch=self.B)
        self._ctx[name] = ctx
        self._out[name] = _Outputs(ctx, self.B, s.d, s.V, self.dev, self.want_logits)
        return ctx

    def _bind(self, ctx: hb.Hydra) -> None:
        ctx.bind_weights(self.arena, self._next_slot)
        self._next_slot += 1

    def ctx(self, name: str) -> hb.Hydra:
        """'main', 'ar' (one-node tree) or 'chainN' (N-token causal chunk), created on demand."""
        if name not in self._ctx:
            parent = [-1] if name == "ar" else chain_parent(int(name[5:]))
            c = self._make_ctx(name, parent)
            self._bind(c)
            need = c.workspace_bytes(self.B)
            if need > self.ws.numel():
                torch.cuda.synchronize()
                self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        return self._ctx[name]

    def add_tree(self, name: str, parent: Sequence[int]) -> hb.Hydra:
        """A further decode context with its own candidate tree on the same weights and cache (the weight arena has
        room for 16 contexts in all)."""
        if name in self._ctx:
            raise ValueError(f"context {name!r} exists")
        c = self._make_ctx(name, list(parent))
        self._bind(c)
        need = c.workspace_bytes(self.B)
        if need > self.ws.numel():
            torch.cuda.synchronize()
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)
        return c

    # ---- prefix-attention contexts (one per chain length) --------------------------
    def _prefix_ctx_new(self, P: int) -> hb.Hydra:
        s = self.shape
        c = hb.Hydra(d=s.d, n_layers=1, n_heads=s.H, head_dim=s.Dh, ffn=s.F, vocab=32, dtype=self.dtype_code,
                     rms_eps=s.rms_eps, rope_theta=s.rope_theta, max_pos=self._max_pos, n_draft_heads=0,
                     mlp_layers=1, include_root_embedding=1, parent=chain_parent(P), max_batch=self.B)
        self._pctx[P] = c
        return c

    def _prefix_bind(self, c: hb.Hydra) -> None:
        c.bind_weights(self.parena, self._pnext_slot)
        self._pnext_slot += 1
        need = c.workspace_bytes(self.B)
        if need > self.ws.numel():
            torch.cuda.synchronize()
            self.ws = torch.empty(need, dtype=torch.uint8, device=self.dev)

    def prefix_ctx(self, P: int) -> hb.Hydra:
        if P not in self._pctx:
            self._prefix_bind(self._prefix_ctx_new(P))
        return self._pctx[P]

    def prefix_attention(self, name: str = "main") -> None:
        """Feeds the accepted tokens' hidden states of context `name` to the prefix layer; h_last becomes its output."""
        c, o = self._ctx[name], self._out[name]
        P = o.path.shape[1]
        self.pkv.seq_len_hint = self.host_len
        self.prefix_ctx(P).hydra_prefix_attention(self.B, self.ws, o.hidden, c.T, o.path, o.n_acc, self.pseq_len, self.pkv, self.h_last)

    def out(self, name: str = "main") -> _Outputs:
        return self._out[name]

    def _load_weights(self, get) -> None:
        s, m = self.shape, self.main
        m.load_tensor(hb.W_EMBED, 0, 0, get("embed"))
        m.load_tensor(hb.W_LM_HEAD, 0, 0, get("lm_head"))
        m.load_tensor(hb.W_FINAL_NORM, 0, 0, get("final_norm"))
        per_layer = (("attn_norm", hb.W_ATTN_NORM), ("wq", hb.W_WQ), ("wk", hb.W_WK), ("wv", hb.W_WV), ("wo", hb.W_WO),
                     ("ffn_norm", hb.W_FFN_NORM), ("w_gate", hb.W_GATE), ("w_up", hb.W_UP), ("w_down", hb.W_DOWN))
        for l in range(s.NL):
            for nm, kind in per_layer:
                m.load_tensor(kind, l, 0, get(f"layers.{l}.{nm}"))
            torch.cuda.synchronize()          # sources may be freed by the provider
        for i in range(1, s.K + 1):
            m.load_tensor(hb.W_HEAD_W1, i, 0, get(f"heads.{i}.w1"))
            m.load_tensor(hb.W_HEAD_B1, i, 0, get(f"heads.{i}.b1"))
            for j in range(2, s.mlp_layers + 1):
                m.load_tensor(hb.W_HEAD_WL, i, j, get(f"heads.{i}.w{j}"))
                m.load_tensor(hb.W_HEAD_BL, i, j, get(f"heads.{i}.b{j}"))
            m.load_tensor(hb.W_HEAD_WOUT, i, 0, get(f"heads.{i}.wout"))
            torch.cuda.synchronize()

    # ---- steps ----------------------------------------------------------------
    def _hint(self, T: int) -> None:
        self.kv.seq_len_hint = self.host_len

    def reset(self) -> None:
        self.seq_len.zero_(); self.h_last.zero_(); self.root.zero_()
        if self.prefix:
            self.pseq_len.zero_()
        self.host_len = 0
        self._len_event = None

    def prefill(self, prompts: torch.Tensor) -> None:
        """prompts: int32 [B, L] (same length for every row).  Causal chunks through
        tree_verify_forward with a chain tree; the state update is kv_compact with the
        identity path."""
        B, L = prompts.shape
        assert B == self.B
        prompts = prompts.to(self.dev, torch.int32)
        pos = 0
        while pos < L:
            n = min(self.prefill_chunk, L - pos)
            name = f"chain{n}"
            c = self.ctx(name)
            o = self._out[name]
            o.tree_tokens.copy_(prompts[:, pos:pos + n])
            self._hint(n)
            c.tree_verify_forward(B, self.ws, o.tree_tokens, self.seq_len, self.kv, o.hidden, o.argmax, o.margin, o.logits)
            o.n_acc.fill_(n)
            o.path.copy_(torch.arange(n, dtype=torch.int32, device=self.dev).expand(B, n))
            o.last_node.fill_(n - 1)
            o.next_root.copy_(o.argmax[:, n - 1])
            c.kv_compact(B, o.n_acc, o.path, o.next_root, o.last_node, o.hidden, self.kv, self.seq_len, self.h_last,
                         self.root, o.kv_index)
            if self.prefix:
                self.prefix_attention(name)           # hint: still the length before this chunk
            pos += n
            self.host_len += n

    def draft(self, name: str = "main") -> None:
        c, o = self.ctx(name), self._out[name]
        c.hydra_draft_tree(self.B, self.ws, self.h_last, self.root, o.tree_tokens)

    def verify(self, name: str = "main") -> None:
        c, o = self.ctx(name), self._out[name]
        self._hint(c.T)
        c.tree_verify_forward(self.B, self.ws, o.tree_tokens, self.seq_len, self.kv, o.hidden, o.argmax, o.margin, o.logits)

    def accept(self, name: str = "main") -> None:
        c, o = self.ctx(name), self._out[name]
        c.accept_greedy(self.B, o.tree_tokens, o.argmax, o.n_acc, o.path, o.next_root, o.last_node)

    def accept_typical(self, tau: float, eps: float, alpha: float, u: Optional[torch.Tensor] = None, name: str = "main") -> None:
        """Typical acceptance instead of greedy acceptance; needs the session to keep logits (want_logits=True)."""
        c, o = self.ctx(name), self._out[name]
        if o.logits is None:
            raise ValueError("typical acceptance needs the logits: create the Session with want_logits=True")
        c.accept_typical(self.B, self.ws, o.tree_tokens, o.logits, tau, eps, alpha, u, o.n_acc, o.path, o.next_root, o.last_node)

    def compact(self, name: str = "main") -> None:
        c, o = self.ctx(name), self._out[name]
        self._hint(c.T)
        c.kv_compact(self.B, o.n_acc, o.path, o.next_root, o.last_node, o.hidden, self.kv, self.seq_len, self.h_last,
                     self.root, o.kv_index)
        self.host_len += c.depth + 1          # upper bound; the device holds the exact value
        self._growth_since_copy += c.depth + 1

    def step(self, name: str = "main", hook=None, typical=None) -> None:
        """One speculative step of every row.  `hook(outputs)` may edit tree_tokens between
        draft and verify (scripted-acceptance experiments).  typical = (tau, eps, alpha, u): the accepted path
        and the next root come from accept_typical (u: device [B] uniform numbers or None) instead of accept_greedy."""
        self._refresh_bound()
        self.draft(name)
        if hook is not None:
            hook(self._out[name])
        self.verify(name)
        if typical is None:
            self.accept(name)
        else:
            self.accept_typical(typical[0], typical[1], typical[2], typical[3], name)
        pre = self.host_len
        self.compact(name)
        if self.prefix:
            post, self.host_len = self.host_len, pre          # the prefix cache is as long as the base cache was before compaction
            self.prefix_attention(name)
            self.host_len = post

    def _refresh_bound(self, every: int = 8) -> None:
        """Asynchronous tightening of the host bound on seq_len: no synchronisation, the value is used when it has arrived."""
        if self._len_event is not None and self._len_event.query():
            self.host_len = min(self.host_len, int(self._len_pinned.max()) + self._growth_since_copy)
            self._len_event = None
        self._steps_since_copy += 1
        if self._len_event is None and self._steps_since_copy >= every:
            self._len_pinned.copy_(self.seq_len, non_blocking=True)
            self._len_event = torch.cuda.Event()
            self._len_event.record()
            self._growth_since_copy = 0
            self._steps_since_copy = 0

    def sync_len(self) -> int:
        """Tighten the host bound from the device (synchronises)."""
        self.host_len = int(self.seq_len.max().item())
        self._len_event = None
        self._steps_since_copy = 0
        return self.host_len

    def generate(self, n_new: int, name: str = "main", max_steps: Optional[int] = None):
        """Runs steps until every row has >= n_new tokens.  Returns (tokens per row, n_acc per step)."""
        self.ctx(name)
        o = self._out[name]
        out = [[] for _ in range(self.B)]
        accs = []
        steps = 0
        while min(len(t) for t in out) < n_new and (max_steps is None or steps < max_steps):
            self.step(name)
            tt, pa, na = o.tree_tokens.cpu(), o.path.cpu(), o.n_acc.cpu()
            for b in range(self.B):
                out[b] += [int(tt[b, pa[b, j]]) for j in range(int(na[b]))]
            accs.append(na.tolist())
            self.sync_len()
            steps += 1
        return [t[:n_new] for t in out], accs
