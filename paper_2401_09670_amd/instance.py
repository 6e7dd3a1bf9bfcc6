"""One serving instance's loop around the per-layer C ABI: a stack of L layers, a paged KV pool, and the
host-side bookkeeping the paper leaves to the serving engine (Sec. 4.3: prefill batches are formed first
come first served up to a token budget near the saturation length L_m; Sec. 3.3 / 4.3: the decoding side
pulls each layer's K/V into its paged memory; Sec. 2.1: decoding runs as one continuously refilled batch,
one token per request per step).

Two halves, deliberately separate:

* ``BlockPool`` / ``Scheduler`` - pure host logic (numpy only): page allocation, first-come-first-served
  prefill batches under a token cap, admission by free pages, the continuously refilled decode batch.
  Testable without a GPU.
* ``GpuStack`` - the device side: L layers of seeded random parameters, embedding tables, the KV pool,
  and the per-phase loops that call ``ds_embed`` -> L x (``ds_prefill`` + ``ds_kv_migrate``) ->
  ``ds_next_token`` and ``ds_embed`` -> L x ``ds_decode_step`` -> ``ds_next_token``.  Every step of the
  arithmetic runs inside the library; this file only sequences calls and owns buffers.

``run_workload`` drives both over a synthetic request list and reports whole-stack prefill tokens/s,
time per output token (mean / P50 / P90 over decoding steps), hand-off GB/s and the roofline fractions
those imply.  On one GPU the two phases are serialised: a prefill batch runs whenever the decode batch has
free rows and the pool has pages, then decoding resumes; each phase is timed on its own with events on the
stream, so the figures are per-phase rates of one instance, not a colocated system's latency.
"""
from __future__ import annotations

import argparse
import collections
import json
import sys
import time
from dataclasses import dataclass, field
from typing import Deque, Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import synth

VOCAB = 50272      # OPT's vocabulary (Sec. 6.1 uses the OPT series)
N_POS = 2048       # OPT's learned position table; longer contexts are clamped by ds_embed


# ---------------------------------------------------------------------------------------------------
# host logic
# ---------------------------------------------------------------------------------------------------
@dataclass
class Request:
    rid: int
    prompt_len: int
    output_len: int            # tokens to generate, the first of which comes out of the prefill pass
    preloaded: bool = False    # context already sits in the pool (decode-only workloads)


class BlockPool:
    """Free list of physical page ids.  Ids are handed out in a seeded shuffled order, so that a sequence's
    pages are scattered the way they are in a pool that has been running for a while."""

    def __init__(self, num_blocks: int, seed: int = 0):
        if num_blocks <= 0:
            raise ValueError("pool needs at least one page")
        self.num_blocks = int(num_blocks)
        self._free = np.random.default_rng(seed).permutation(self.num_blocks).astype(np.int32)
        self._n = self.num_blocks

    @property
    def n_free(self) -> int:
        return self._n

    def alloc(self, n: int) -> np.ndarray:
        if n < 0 or n > self._n:
            raise MemoryError(f"asked for {n} pages, {self._n} free")
        out = self._free[self._n - n:self._n].copy()
        self._n -= n
        return out

    def free(self, ids: Sequence[int]) -> None:
        ids = np.asarray(ids, dtype=np.int32)
        if self._n + len(ids) > self.num_blocks:
            raise RuntimeError("more pages returned than were handed out")
        self._free[self._n:self._n + len(ids)] = ids
        self._n += len(ids)


@dataclass
class _Seq:
    req: Request
    ctx_len: int                # tokens whose K/V sit in the pool
    steps_left: int             # decoding steps still to run
    blocks: List[int] = field(default_factory=list)
    reserved: int = 0           # pages promised to this sequence and not yet taken


class Scheduler:
    """Which requests run in which phase, and where their pages are.

    A request moves waiting -> (prefill batch) -> ready -> decode row -> finished.  `ready` holds requests
    whose prompt has been processed and whose K/V already sit in pool pages but which have no decode row yet:
    the prefill side works ahead of the decoding side and its memory is the buffer between them (Sec. 4.3),
    which is what lets prefill batches fill up to the token cap instead of trickling in one request per freed
    row.  The prefill side runs one more batch whenever that buffer is empty.

    Memory policy (the paper fixes none beyond paged allocation): a request is admitted to a prefill batch
    only when the pool can hold its whole life (prompt + generated tokens); the pages for the prompt are taken
    then and one more each time decoding crosses a page boundary, out of that reservation - so decoding never
    stalls or evicts.  A synthetic request's output length is known in advance; a live system would reserve
    its maximum.
    """

    def __init__(self, requests: Sequence[Request], pool: BlockPool, max_batch: int, token_cap: int,
                 block_size: int = 16, max_blocks_per_seq: Optional[int] = None):
        self.pool, self.bs = pool, int(block_size)
        self.max_batch, self.token_cap = int(max_batch), int(token_cap)
        self.waiting: Deque[Request] = collections.deque(requests)
        self.ready: Deque[_Seq] = collections.deque()
        longest = max((r.prompt_len + max(r.output_len - 1, 0) for r in requests), default=1)
        self.max_blocks = int(max_blocks_per_seq or synth.blocks_needed(longest, self.bs))
        self.active: Dict[int, _Seq] = {}
        self._free_rows = list(range(self.max_batch - 1, -1, -1))
        self._promised = 0          # pages reserved by admitted sequences and not yet taken from the pool
        self.finished: List[int] = []
        for r in requests:
            if self._life_blocks(r) > min(self.max_blocks, pool.num_blocks):
                raise ValueError(f"request {r.rid} can never fit ({self._life_blocks(r)} pages)")

    def _life_blocks(self, r: Request) -> int:
        return synth.blocks_needed(r.prompt_len + max(r.output_len - 1, 0), self.bs)

    @property
    def done(self) -> bool:
        return not self.waiting and not self.ready and not self.active

    def next_prefill_batch(self) -> List[_Seq]:
        """When nothing prefilled is waiting for a row: takes requests from the head of the queue (no
        skipping: first come first served) while the pool can hold the request's whole life and the batch
        stays within the token cap (a prompt longer than the cap runs alone), allocates the prompts' pages and
        puts the requests on `ready`.  Preloaded requests pass through the same way in batches of their own
        (their prompt is not run; the caller fills their pages)."""
        batch: List[_Seq] = []
        if self.ready:
            return batch
        tokens = 0
        while self.waiting:
            r = self.waiting[0]
            if batch and r.preloaded != batch[0].req.preloaded:
                break
            if not r.preloaded and batch and tokens + r.prompt_len > self.token_cap:
                break
            if r.preloaded and len(batch) >= self.max_batch:
                break
            life = self._life_blocks(r)
            if self.pool.n_free - self._promised < life:
                break
            self.waiting.popleft()
            now = synth.blocks_needed(r.prompt_len, self.bs)
            seq = _Seq(r, r.prompt_len, max(r.output_len - 1, 0), list(self.pool.alloc(now)), life - now)
            self._promised += seq.reserved
            batch.append(seq)
            tokens += 0 if r.preloaded else r.prompt_len
        self.ready.extend(batch)
        return batch

    def _release(self, s: _Seq) -> None:
        self.pool.free(s.blocks)
        self._promised -= s.reserved
        self.finished.append(s.req.rid)

    def place_ready(self) -> List[Tuple[int, int]]:
        """Moves prefilled requests into free decode rows, oldest first; a request that wanted a single token
        is complete after its prefill pass and leaves without taking a row.  Returns [(row, request id)]."""
        placed = []
        while self.ready and (self._free_rows or self.ready[0].steps_left == 0):
            s = self.ready.popleft()
            if s.steps_left == 0:
                self._release(s)
                continue
            row = self._free_rows.pop()
            self.active[row] = s
            placed.append((row, s.req.rid))
        return placed

    def retire_finished(self) -> List[int]:
        """Frees the rows and pages of requests that have no decoding step left.  Returns their ids."""
        out = []
        for row in [w for w, s in self.active.items() if s.steps_left == 0]:
            s = self.active.pop(row)
            self._release(s)
            self._free_rows.append(row)
            out.append(s.req.rid)
        return out

    def decode_rows(self) -> List[int]:
        return sorted(self.active)

    def prepare_step(self, rows: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
        """Context lengths before the step and the page table for it; takes the page the step's new token
        needs when it starts one."""
        ctx = np.empty(len(rows), dtype=np.int32)
        table = np.full((len(rows), self.max_blocks), -1, dtype=np.int32)
        for i, row in enumerate(rows):
            s = self.active[row]
            if s.ctx_len == len(s.blocks) * self.bs:
                if s.reserved <= 0:
                    raise RuntimeError("sequence outgrew its reservation")
                s.blocks.append(int(self.pool.alloc(1)[0]))
                s.reserved -= 1
                self._promised -= 1
            ctx[i] = s.ctx_len
            table[i, :len(s.blocks)] = s.blocks
        return ctx, table

    def prefill_table(self, batch: Sequence[_Seq]) -> np.ndarray:
        table = np.full((len(batch), self.max_blocks), -1, dtype=np.int32)
        for i, s in enumerate(batch):
            table[i, :len(s.blocks)] = s.blocks
        return table

    def finish_step(self, rows: Sequence[int]) -> None:
        for row in rows:
            s = self.active[row]
            s.ctx_len += 1
            s.steps_left -= 1


# ---------------------------------------------------------------------------------------------------
# algorithmic work, for the roofline fractions of the report
# ---------------------------------------------------------------------------------------------------
def prefill_flops(lens: Sequence[int], shape: synth.ModelShape, n_layers: int, vocab: int) -> float:
    """2 t (h qkv + h^2 + 2 h m) GEMM flops + causal attention 2 h sum(l^2) per layer (App. A.2, true
    flops = 2 x the multiply-accumulate counts printed there), + the vocabulary GEMM for one row per prompt."""
    h, m = shape.hidden, shape.ffn
    t = float(sum(lens))
    t2 = float(sum(int(l) * int(l) for l in lens))
    per_layer = 2.0 * t * (h * shape.qkv_width + h * h + 2 * h * m) + 2.0 * h * t2
    return n_layers * per_layer + 2.0 * len(lens) * h * vocab


def decode_bytes(ctx_lens: Sequence[int], shape: synth.ModelShape, n_layers: int, vocab: int) -> float:
    """Weights once + K and V of every cached token (incl. the new one) once + activations (App. A.3),
    per layer, + the vocabulary matrix once."""
    h, m = shape.hidden, shape.ffn
    B = len(ctx_lens)
    kvw = shape.kv_heads * shape.head_dim
    weights = 2.0 * (h * shape.qkv_width + h * h + 2 * h * m)
    kv = 2.0 * 2.0 * kvw * float(sum(int(c) + 1 for c in ctx_lens))
    act = 2.0 * (8 * B * h + 2 * B * m) + 2.0 * 2 * B * kvw
    return n_layers * (weights + kv + act) + 2.0 * h * vocab


# ---------------------------------------------------------------------------------------------------
# device side
# ---------------------------------------------------------------------------------------------------
class GpuStack:
    """L layers + token tables + KV pool on cuda:0, and the two phase loops."""

    def __init__(self, shape: synth.ModelShape, n_layers: int, seed: int, pool_blocks: int, max_batch: int,
                 max_prefill_tokens: int, max_ctx: int, max_blocks_per_seq: int, vocab: int = VOCAB,
                 n_pos: int = N_POS, max_requests: int = 4096, overlap_handoff: bool = False, log=lambda s: None,
                 pool_layers: Optional[int] = None):
        import torch
        from . import binding
        if not torch.cuda.is_available():
            raise RuntimeError("GpuStack needs a GPU")
        self.torch, self.shape, self.L = torch, shape, int(n_layers)
        self.dev = torch.device("cuda:0")
        self.vocab, self.n_pos = int(vocab), int(n_pos)
        self.max_batch, self.max_blocks = int(max_batch), int(max_blocks_per_seq)
        self.max_ctx = int(max_ctx)
        h, m, s = shape.hidden, shape.ffn, shape.head_dim
        self.kvw = shape.kv_heads * s
        self.gen = torch.Generator(device="cuda")
        self.gen.manual_seed(int(seed))
        self.ctx = binding.Context(h, shape.n_heads, s, m, shape.block_size, shape.ln_eps, shape.n_kv_heads)

        self.layers = []
        self._keep = []
        for li in range(self.L):
            w = {"ln1_g": self._nrm((h,), 0.02, 1.0), "ln1_b": self._nrm((h,), 0.02),
                 "w_qkv": self._nrm((shape.qkv_width, h), 0.02), "b_qkv": self._nrm((shape.qkv_width,), 0.02),
                 "w_o": self._nrm((h, h), 0.02), "b_o": self._nrm((h,), 0.02),
                 "ln2_g": self._nrm((h,), 0.02, 1.0), "ln2_b": self._nrm((h,), 0.02),
                 "w_fc1": self._nrm((m, h), 0.02), "b_fc1": self._nrm((m,), 0.02),
                 "w_fc2": self._nrm((h, m), 0.02), "b_fc2": self._nrm((h,), 0.02)}
            lw, keep = self.ctx.pack_weights(w)
            self.layers.append(lw)
            self._keep.append(keep)
            if (li + 1) % 8 == 0 or li + 1 == self.L:
                log(f"weights: {li + 1}/{self.L} layers on the device")
        # OPT ties the output matrix to the token table
        self.tok_emb = self._nrm((self.vocab, h), 0.02)
        self.pos_emb = self._nrm((self.n_pos, h), 0.02)
        self.lnf_g, self.lnf_b = self._nrm((h,), 0.02, 1.0), self._nrm((h,), 0.02)

        self.num_blocks = int(pool_blocks)
        # pool_layers < L is the timing-only mode: layer li uses the pool of layer li % pool_layers, so a batch
        # whose KV does not fit beside the weights can still be stepped through the whole stack at its true
        # shape.  Every kernel does the work it would do, the cache contents (and so the outputs) are meaningless.
        self.pool_layers = int(pool_layers or self.L)
        pool_shape = (self.pool_layers, self.num_blocks, shape.kv_heads, shape.block_size, s)
        self.k_pool = torch.empty(pool_shape, dtype=torch.bfloat16, device=self.dev)
        self.v_pool = torch.empty(pool_shape, dtype=torch.bfloat16, device=self.dev)

        T = int(max_prefill_tokens)
        self.max_prefill_tokens = T
        bf = dict(dtype=torch.bfloat16, device=self.dev)
        self.xa, self.xb = torch.empty((max(T, 1), h), **bf), torch.empty((max(T, 1), h), **bf)
        # One layer's contiguous K/V at a time (the hand-off is per layer, Sec. 3.3); two pairs when the hand-off
        # of layer i runs on a second stream beside the compute of layer i+1.
        self.overlap_handoff = bool(overlap_handoff)
        self.kv_out = [(torch.empty((max(T, 1), self.kvw), **bf), torch.empty((max(T, 1), self.kvw), **bf))
                       for _ in range(2 if self.overlap_handoff else 1)]
        self.handoff_stream = torch.cuda.Stream() if self.overlap_handoff else None   # default priority
        self.ws_prefill = torch.empty(max(self.ctx.ds_prefill_workspace_bytes(T), 256) if T else 256,
                                      dtype=torch.uint8, device=self.dev)
        self.da, self.db = torch.empty((self.max_batch, h), **bf), torch.empty((self.max_batch, h), **bf)
        self.ws_decode = torch.empty(max(self.ctx.ds_decode_workspace_bytes(self.max_batch, self.max_ctx), 256),
                                     dtype=torch.uint8, device=self.dev)
        self.ws_next = torch.empty(max(self.ctx.ds_next_token_workspace_bytes(256, self.vocab), 256),
                                   dtype=torch.uint8, device=self.dev)
        self.cur_tok = torch.zeros(self.max_batch, dtype=torch.int32, device=self.dev)      # per decode row
        self.first_tok = torch.zeros(int(max_requests), dtype=torch.int32, device=self.dev)  # per request id
        self.next_tok = torch.empty(256, dtype=torch.int32, device=self.dev)   # ds_next_token takes <= 256 rows
        # Tests set this to {layer: []}: copies of those layers' inputs and outputs are appended per call
        # (for a decoding step also the layer's pool as the step leaves it).
        self.capture = None

    def _nrm(self, shape, std, mean=0.0):
        t = self.torch.empty(shape, dtype=self.torch.float32, device=self.dev)
        t.normal_(mean, std, generator=self.gen)
        return t.to(self.torch.bfloat16)

    def _i32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.dev)

    def _event(self):
        e = self.torch.cuda.Event(enable_timing=True)
        e.record()
        return e

    def fill_pool_pages(self, pages: Sequence[int]) -> None:
        """Seeded N(0,1) K/V in the given pages of every layer (decode-only workloads whose contexts were
        not produced by a prefill here)."""
        idx = self._i32(pages).long()
        bs, s, nk = self.shape.block_size, self.shape.head_dim, self.shape.kv_heads
        for pool in (self.k_pool, self.v_pool):
            for li in range(self.pool_layers):
                blk = self.torch.empty((len(pages), nk, bs, s), dtype=self.torch.bfloat16, device=self.dev)
                blk.normal_(0.0, 1.0, generator=self.gen)
                pool[li].index_copy_(0, idx, blk)

    # ---- prefill phase: embed -> L x (layer, hand-off) -> first token of every prompt ----
    def prefill(self, lens: Sequence[int], rids: Sequence[int], table: np.ndarray):
        """Runs one packed batch of prompts (synthetic token ids) through the stack, moves each layer's K/V
        into the pool pages of `table`, and leaves every prompt's first generated token in first_tok[rids].
        Returns (start, end) events of the whole batch and the per-layer (start, end) events of the hand-off."""
        torch = self.torch
        B, t, mx = len(lens), int(sum(lens)), int(max(lens))
        if t > self.max_prefill_tokens:
            raise ValueError(f"batch of {t} tokens exceeds the buffers ({self.max_prefill_tokens})")
        cu_h = synth.cu_seqlens(lens)
        cu = self._i32(cu_h)
        ids = torch.randint(0, self.vocab, (t,), dtype=torch.int32, device=self.dev, generator=self.gen)
        pos = self._i32(np.concatenate([np.arange(l, dtype=np.int32) for l in lens]))
        bt = self._i32(table)
        last = self._i32(cu_h[1:] - 1)
        rids_d = self._i32(rids).long()
        x, y = self.xa[:t], self.xb[:t]
        main = torch.cuda.current_stream()
        start = self._event()
        self.ctx.ds_embed(ids, pos, self.tok_emb, self.vocab, self.pos_emb, self.n_pos, t, x)
        mig = []
        for li in range(self.L):
            k_out, v_out = (b[:t] for b in self.kv_out[li % len(self.kv_out)])
            if self.overlap_handoff and li >= 2:
                main.wait_event(mig[li - 2][1])      # the hand-off that last read this K/V pair has finished
            self.ctx.ds_prefill(self.layers[li], x, cu, B, t, mx, y, k_out, v_out, self.ws_prefill)
            if self.overlap_handoff:
                # layer li's K/V move into the pool on the second stream while layer li+1 computes
                ready = self._event()
                with torch.cuda.stream(self.handoff_stream):
                    self.handoff_stream.wait_event(ready)
                    a = self._event()
                    self.ctx.ds_kv_migrate(k_out, v_out, cu, B, t, mx, bt, table.shape[1], self.k_pool[li % self.pool_layers],
                                           self.v_pool[li % self.pool_layers], self.num_blocks)
                    mig.append((a, self._event()))
            else:
                a = self._event()
                self.ctx.ds_kv_migrate(k_out, v_out, cu, B, t, mx, bt, table.shape[1], self.k_pool[li % self.pool_layers],
                                       self.v_pool[li % self.pool_layers], self.num_blocks)
                mig.append((a, self._event()))
            if self.capture is not None and li in self.capture:
                self.capture[li].append(dict(kind="prefill", lens=list(lens), x=x.clone(), y=y.clone(),
                                             k_out=k_out.clone(), v_out=v_out.clone()))
            x, y = y, x
        if self.overlap_handoff:
            for a, b in mig[-2:]:
                main.wait_event(b)                   # the pool is complete before anything that follows
        for c0 in range(0, B, 256):
            n = min(256, B - c0)
            self.ctx.ds_next_token(x, last[c0:c0 + n], n, self.lnf_g, self.lnf_b, self.tok_emb, self.vocab,
                                   self.next_tok, None, self.ws_next)
            self.first_tok.index_copy_(0, rids_d[c0:c0 + n], self.next_tok[:n])
        end = self._event()
        return (start, end), mig

    def place(self, placed: Sequence[Tuple[int, int]]) -> None:
        """Requests enter decode rows: cur_tok[row] = the first token their prefill pass produced."""
        if not placed:
            return
        rows = self._i32([row for row, _ in placed]).long()
        rids = self._i32([rid for _, rid in placed]).long()
        self.cur_tok.index_copy_(0, rows, self.first_tok.index_select(0, rids))

    # ---- decoding phase: one token for every active row ----
    def decode_step(self, rows: Sequence[int], ctx_lens: np.ndarray, table: np.ndarray):
        """The token in cur_tok[rows] enters the stack at position ctx_lens, its K/V are appended, and the next
        token replaces it.  Returns (start, end) events."""
        B = len(rows)
        if B > 256:
            raise ValueError("decode batch above 256 rows")
        rows_d = self._i32(rows).long()
        cl = self._i32(ctx_lens)
        bt = self._i32(table)
        max_ctx = int(ctx_lens.max()) + 1
        if max_ctx > self.max_ctx:
            raise ValueError(f"context {max_ctx} exceeds the workspace ({self.max_ctx})")
        ids = self.cur_tok.index_select(0, rows_d)
        x, y = self.da[:B], self.db[:B]
        start = self._event()
        self.ctx.ds_embed(ids, cl, self.tok_emb, self.vocab, self.pos_emb, self.n_pos, B, x)
        for li in range(self.L):
            self.ctx.ds_decode_step(self.layers[li], x, cl, bt, B, table.shape[1], max_ctx, self.k_pool[li % self.pool_layers],
                                    self.v_pool[li % self.pool_layers], self.num_blocks, y, self.ws_decode)
            if self.capture is not None and li in self.capture:
                self.capture[li].append(dict(kind="decode", ctx=np.array(ctx_lens), table=np.array(table),
                                             x=x.clone(), y=y.clone(), k_pool=self.k_pool[li % self.pool_layers].clone(),
                                             v_pool=self.v_pool[li % self.pool_layers].clone()))
            x, y = y, x
        self.ctx.ds_next_token(x, None, B, self.lnf_g, self.lnf_b, self.tok_emb, self.vocab, self.next_tok, None,
                               self.ws_next)
        end = self._event()
        self.cur_tok.index_copy_(0, rows_d, self.next_tok[:B])
        return start, end


# ---------------------------------------------------------------------------------------------------
# driver
# ---------------------------------------------------------------------------------------------------
def run_workload(stack: GpuStack, sched: Scheduler, max_steps: Optional[int] = None, log=lambda s: None) -> dict:
    """Runs the scheduler's requests to completion (or for max_steps decoding steps) and returns raw timings:
    per prefill batch (lens, ms, hand-off ms) and per decoding step (context lengths, ms)."""
    torch = stack.torch
    prefills, steps = [], []
    pending_p, pending_s = [], []

    def drain():
        torch.cuda.synchronize()
        for lens, (a, b), mig in pending_p:
            prefills.append(dict(lens=lens, ms=a.elapsed_time(b), migrate_ms=sum(x.elapsed_time(y) for x, y in mig),
                                 overlapped=stack.overlap_handoff))
        for ctx, (a, b) in pending_s:
            steps.append(dict(batch=len(ctx), kv_tokens=int(ctx.sum()) + len(ctx), ctx=ctx, ms=a.elapsed_time(b)))
        pending_p.clear()
        pending_s.clear()

    t0 = time.time()
    last_log = t0
    n_steps = 0
    while not sched.done:
        progressed = True
        while progressed:
            n_done = len(sched.finished)
            placed = sched.place_ready()
            stack.place(placed)
            batch = sched.next_prefill_batch()
            if batch and batch[0].req.preloaded:
                stack.fill_pool_pages([p for s in batch for p in s.blocks])
            elif batch:
                lens = [s.req.prompt_len for s in batch]
                ev, mig = stack.prefill(lens, [s.req.rid for s in batch], sched.prefill_table(batch))
                pending_p.append((lens, ev, mig))
            progressed = bool(placed) or bool(batch) or len(sched.finished) != n_done
        rows = sched.decode_rows()
        if not rows:
            if sched.waiting or sched.ready:
                raise RuntimeError("no request fits the pool")
            break
        ctx, table = sched.prepare_step(rows)
        pending_s.append((ctx, stack.decode_step(rows, ctx, table)))
        sched.finish_step(rows)
        sched.retire_finished()
        n_steps += 1
        if len(pending_s) >= 64:
            drain()
        if time.time() - last_log > 20:
            last_log = time.time()
            log(f"step {n_steps}: {len(sched.finished)} requests finished, {len(sched.waiting)} waiting, "
                f"{len(sched.ready)} prefilled, {len(rows)} in the batch, {sched.pool.n_free} pages free")
        if max_steps is not None and n_steps >= max_steps:
            break
    drain()
    return dict(prefills=prefills, steps=steps, wall_s=time.time() - t0, finished=len(sched.finished))


def summarise(raw: dict, shape: synth.ModelShape, n_layers: int, vocab: int = VOCAB) -> dict:
    """Rates and roofline fractions from run_workload's timings."""
    out = dict(finished=raw["finished"], wall_s=raw["wall_s"])
    P = raw["prefills"]
    if P:
        tok = sum(sum(p["lens"]) for p in P)
        # serial hand-off: its time is taken out of the prefill figure; overlapped: it hides inside it
        ms = sum(p["ms"] - (0.0 if p.get("overlapped") else p["migrate_ms"]) for p in P)
        fl = sum(prefill_flops(p["lens"], shape, n_layers, vocab) for p in P)
        mig_bytes = sum(2.0 * 2 * 2 * shape.kv_heads * shape.head_dim * sum(p["lens"]) for p in P) * n_layers
        mig_ms = sum(p["migrate_ms"] for p in P)
        out["prefill"] = dict(batches=len(P), prompts=sum(len(p["lens"]) for p in P), tokens=tok, ms=ms,
                              tokens_per_s=tok / (ms * 1e-3), tflops=fl / (ms * 1e-3) / 1e12,
                              mfma_frac=fl / (ms * 1e-3) / 2.5e15,
                              mean_batch_tokens=tok / len(P))
        out["migrate"] = dict(bytes=mig_bytes, ms=mig_ms, gb_per_s=mig_bytes / (mig_ms * 1e-3) / 1e9,
                              hbm_frac=mig_bytes / (mig_ms * 1e-3) / 8e12, overlapped=bool(P[0].get("overlapped")))
    S = raw["steps"]
    if S:
        ms = np.array([s["ms"] for s in S])
        by = np.array([decode_bytes(s["ctx"], shape, n_layers, vocab) for s in S])
        out["decode"] = dict(steps=len(S), tokens=int(sum(s["batch"] for s in S)),
                             mean_batch=float(np.mean([s["batch"] for s in S])),
                             mean_ctx=float(np.sum([s["kv_tokens"] for s in S]) / np.sum([s["batch"] for s in S])),
                             tpot_ms_mean=float(ms.mean()), tpot_ms_p50=float(np.percentile(ms, 50)),
                             tpot_ms_p90=float(np.percentile(ms, 90)), tpot_ms_max=float(ms.max()),
                             tokens_per_s=float(sum(s["batch"] for s in S) / (ms.sum() * 1e-3)),
                             gb_per_s=float(by.sum() / (ms.sum() * 1e-3) / 1e9),
                             hbm_frac=float(by.sum() / (ms.sum() * 1e-3) / 8e12))
        top = max(s["batch"] for s in S)
        full = np.array([s["batch"] == top for s in S])
        out["decode_full_batch"] = dict(batch=int(top), steps=int(full.sum()), tpot_ms_mean=float(ms[full].mean()),
                                        tpot_ms_p90=float(np.percentile(ms[full], 90)),
                                        mean_ctx=float(np.mean([s["kv_tokens"] / s["batch"] for s, f in zip(S, full) if f])),
                                        tokens_per_s=float(top * full.sum() / (ms[full].sum() * 1e-3)),
                                        hbm_frac=float(by[full].sum() / (ms[full].sum() * 1e-3) / 8e12))
    return out


def requests_for(cfg: dict, count: int) -> List[Request]:
    """The synthetic request list of a workload recipe (synth.config): lengths only, seeded."""
    seed = cfg["seed"]
    if "prompt" in cfg:
        p, o = cfg["prompt"], cfg["output"]
        if p["kind"] == "lognormal":
            pl = synth.lognormal_lengths(count, p["median"], p["sigma"], p["lo"], p["hi"], seed)
            ol = synth.lognormal_lengths(count, o["median"], o["sigma"], o["lo"], o["hi"], seed, stream=1)
        else:
            pl = synth.uniform_lengths(count, p["lo"], p["hi"], seed)
            ol = synth.uniform_lengths(count, o["lo"], o["hi"], seed, stream=1)
        return [Request(i, int(pl[i]), int(ol[i])) for i in range(count)]
    reqs = [Request(i, int(l), 1) for i, l in enumerate(cfg["prefill_lens"])]
    c = cfg["decode_ctx"]
    ctx = synth.uniform_lengths(cfg["decode_batch"], c["lo"], c["hi"], seed)
    reqs += [Request(len(reqs) + i, int(l), cfg["decode_steps"] + 1, preloaded=True) for i, l in enumerate(ctx)]
    return reqs


def plan_for(cfg: dict, reqs: Sequence[Request], pool_gb: float) -> dict:
    """Buffer and pool sizes for a request list: the pool takes pool_gb of memory or what the whole list
    needs at once, whichever is smaller."""
    shape, L, bs = cfg["shape"], cfg["layers"], cfg["shape"].block_size
    life = [synth.blocks_needed(r.prompt_len + max(r.output_len - 1, 0), bs) for r in reqs]
    page_bytes = 2 * 2 * shape.kv_heads * shape.head_dim * bs * L
    blocks = min(int(pool_gb * 1e9 // page_bytes), int(sum(life)))
    cap = cfg.get("prefill_token_cap") or max(sum(cfg.get("prefill_lens", [0])), max(r.prompt_len for r in reqs))
    longest_prompt = max((r.prompt_len for r in reqs if not r.preloaded), default=0)
    return dict(pool_blocks=max(blocks, max(life)), page_bytes=page_bytes, token_cap=int(cap),
                max_prefill_tokens=int(max(cap, longest_prompt)), max_blocks=int(max(life)),
                max_ctx=int(max(life)) * bs, max_batch=int(cfg["decode_batch"]))


def timing_only_decode(cfg: dict, batch: int, steps: int, pool_gb: float, log=lambda s: None) -> dict:
    """TIMING ONLY - the outputs of this run mean nothing.  Steps a decode batch of `batch` requests through the
    whole stack at the contexts the workload recipe gives (prompt + a seeded share of the output already
    generated), with every layer's weights resident but KV pools for only as many layers as fit `pool_gb`;
    layer li reads and appends to the pool of layer li % pool_layers.  Each kernel streams the bytes it would
    stream with a full set of pools (a layer's pool is far larger than the last-level cache, so re-using it a
    few layers later gives no cache hits), which is what the time per output token depends on."""
    import torch
    shape, L, bs = cfg["shape"], cfg["layers"], cfg["shape"].block_size
    p, o, seed = cfg["prompt"], cfg["output"], cfg["seed"]
    draw = synth.lognormal_lengths if p["kind"] == "lognormal" else None
    if draw:
        pl = synth.lognormal_lengths(batch, p["median"], p["sigma"], p["lo"], p["hi"], seed, stream=10)
        ol = synth.lognormal_lengths(batch, o["median"], o["sigma"], o["lo"], o["hi"], seed, stream=11)
    else:
        pl = synth.uniform_lengths(batch, p["lo"], p["hi"], seed, stream=10)
        ol = synth.uniform_lengths(batch, o["lo"], o["hi"], seed, stream=11)
    frac = np.random.Generator(np.random.Philox(key=[seed, 7012])).random(batch)
    ctx0 = (pl + np.floor(frac * np.maximum(ol - 1, 0))).astype(np.int32)      # tokens cached when timing starts
    cap = ctx0 + steps
    table, nblk = synth.make_block_tables([int(c) for c in cap], bs, seed)
    layer_bytes = 2 * 2 * shape.kv_heads * shape.head_dim * bs * nblk
    pool_layers = int(max(1, min(L, pool_gb * 1e9 // layer_bytes)))
    log(f"timing-only: batch {batch}, contexts {int(ctx0.min())}..{int(ctx0.max())} (mean {ctx0.mean():.0f}), "
        f"{nblk} pages = {layer_bytes / 1e9:.2f} GB per layer, pools for {pool_layers} of {L} layers")
    stack = GpuStack(shape, L, seed, nblk, batch, 0, int(cap.max()) + 1, table.shape[1], max_requests=batch,
                     log=log, pool_layers=pool_layers)
    stack.k_pool.normal_(0.0, 1.0, generator=stack.gen)
    stack.v_pool.normal_(0.0, 1.0, generator=stack.gen)
    stack.cur_tok.copy_(torch.randint(0, stack.vocab, (batch,), generator=stack.gen, device=stack.dev,
                                      dtype=torch.int32))
    rows = list(range(batch))
    ev = []
    for j in range(steps + 2):                                   # two untimed steps first
        ev.append((ctx0 + max(j - 2, 0), stack.decode_step(rows, ctx0 + max(j - 2, 0), table)))
    torch.cuda.synchronize()
    S = [dict(batch=batch, kv_tokens=int(c.sum()) + batch, ctx=c, ms=a.elapsed_time(b)) for c, (a, b) in ev[2:]]
    res = summarise(dict(prefills=[], steps=S, wall_s=0.0, finished=0), shape, L)["decode"]
    res.update(pool_layers=pool_layers, layers=L, layer_kv_gb=layer_bytes / 1e9, ctx_min=int(ctx0.min()),
               ctx_max=int(ctx0.max()))
    return res


def timing_only_markdown(cfg: dict, r: dict, cmd: str) -> str:
    return "\n".join([
        f"## Timing-only: decode batch {int(r['mean_batch'])} through all {r['layers']} layers (outputs meaningless)", "",
        f"Produced by `{cmd}`.  The KV of this batch ({r['layer_kv_gb']:.2f} GB per layer, "
        f"{r['layer_kv_gb'] * r['layers']:.0f} GB over the stack) does not fit beside the weights; layer li uses the "
        f"pool of layer li mod {r['pool_layers']} (random contents).  Every kernel runs at its true shape and streams "
        "its true byte count; only the cache contents, hence the generated tokens, are meaningless.", "",
        "| decoding (timing only) | value |", "|---|---|",
        f"| steps / contexts | {r['steps']} / {r['ctx_min']}..{r['ctx_max']}, mean {r['mean_ctx']:.0f} |",
        f"| time per output token (one whole-stack step) | **mean {r['tpot_ms_mean']:.2f} ms**, P50 "
        f"{r['tpot_ms_p50']:.2f}, P90 {r['tpot_ms_p90']:.2f} |",
        f"| decode rate | {r['tokens_per_s']:.0f} tokens/s |",
        f"| algorithmic HBM rate | {r['gb_per_s']:.0f} GB/s = {100 * r['hbm_frac']:.1f} % of HBM peak |", ""])


def to_markdown(cfg: dict, plan: dict, n_req: int, res: dict, cmd: str) -> str:
    shape, L = cfg["shape"], cfg["layers"]
    lines = [f"# Whole-stack run: {cfg['name']} ({L} layers, h = {shape.hidden}, {shape.n_heads} x {shape.head_dim}, "
             f"m = {shape.ffn}) on one MI355X", "",
             f"Produced by `{cmd}`; random parameters, synthetic requests (lengths from the seeded recipe, token ids "
             "random, generation greedy through the tied vocabulary matrix).", "",
             f"{n_req} requests; decode batch up to {plan['max_batch']}; prefill batches first come first served up to "
             f"{plan['token_cap']} tokens; KV pool {plan['pool_blocks']} pages of 16 tokens = "
             f"{plan['pool_blocks'] * plan['page_bytes'] / 1e9:.1f} GB over all layers; admission reserves a request's "
             "whole life in pages. Phases are serialised on the one GPU and timed separately.", ""]
    if "prefill" in res:
        p, g = res["prefill"], res["migrate"]
        lines += ["| prefill | value |", "|---|---|",
                  f"| batches / prompts / tokens | {p['batches']} / {p['prompts']} / {p['tokens']} |",
                  f"| mean tokens per batch | {p['mean_batch_tokens']:.0f} |",
                  f"| whole-stack prefill rate | **{p['tokens_per_s']:.0f} tokens/s** |",
                  f"| arithmetic rate | {p['tflops']:.0f} TFLOP/s = {100 * p['mfma_frac']:.1f} % of the bf16 MFMA peak |",
                  f"| hand-off (all layers{', on a second stream beside the next layer: inside the prefill time above' if g.get('overlapped') else ''}) | "
                  f"{g['bytes'] / 1e9:.2f} GB read+written in {g['ms']:.1f} ms = "
                  f"{g['gb_per_s']:.0f} GB/s = {100 * g['hbm_frac']:.1f} % of HBM peak |", ""]
    if "decode" in res:
        d = res["decode"]
        lines += ["| decoding | value |", "|---|---|",
                  f"| steps / tokens generated | {d['steps']} / {d['tokens']} |",
                  f"| mean batch / mean context | {d['mean_batch']:.1f} / {d['mean_ctx']:.0f} |",
                  f"| time per output token (one whole-stack step) | **mean {d['tpot_ms_mean']:.2f} ms**, P50 "
                  f"{d['tpot_ms_p50']:.2f}, P90 {d['tpot_ms_p90']:.2f}, max {d['tpot_ms_max']:.2f} |",
                  f"| decode rate | {d['tokens_per_s']:.0f} tokens/s |",
                  f"| algorithmic HBM rate | {d['gb_per_s']:.0f} GB/s = {100 * d['hbm_frac']:.1f} % of HBM peak |"]
        f = res["decode_full_batch"]
        lines += [f"| steps at the largest batch ({f['batch']}) | {f['steps']} steps, mean context {f['mean_ctx']:.0f}: mean "
                  f"{f['tpot_ms_mean']:.2f} ms, P90 {f['tpot_ms_p90']:.2f} ms, {f['tokens_per_s']:.0f} tokens/s, "
                  f"{100 * f['hbm_frac']:.1f} % of HBM peak |", ""]
    lines += [f"Requests finished: {res['finished']}; wall time of the loop {res['wall_s']:.1f} s "
              "(includes host bookkeeping and the pauses for reading the timers)."]
    return "\n".join(lines) + "\n"


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description="whole-stack run of one serving instance on one GPU")
    ap.add_argument("--config", type=int, default=3, choices=[3, 4, 5], help="workload number (1-based)")
    ap.add_argument("--requests", type=int, default=0, help="requests to draw (0 = a default per workload)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers")
    ap.add_argument("--pool-gb", type=float, default=0.0, help="KV pool size (0 = 160 GB, or less beside large weights)")
    ap.add_argument("--max-steps", type=int, default=0)
    ap.add_argument("--overlap-handoff", action="store_true",
                    help="run each layer's KV hand-off on a second stream beside the next layer's prefill")
    ap.add_argument("--out", type=str, default="")
    ap.add_argument("--timing-only-batch", type=int, default=0,
                    help="TIMING ONLY: step a decode batch of this size through the whole stack with KV pools for as "
                         "many layers as fit (layers share pools; outputs are meaningless), instead of the workload")
    a = ap.parse_args(argv)
    cfg = dict(synth.config(a.config - 1))
    if a.layers:
        cfg["layers"] = a.layers
    if a.timing_only_batch:
        sh, Lt = cfg["shape"], cfg["layers"]
        wgb = Lt * 2.0 * (sh.hidden * sh.qkv_width + sh.hidden ** 2 + 2 * sh.hidden * sh.ffn) / 1e9
        r = timing_only_decode(cfg, a.timing_only_batch, a.max_steps or 16, a.pool_gb or max(8.0, 250.0 - wgb),
                               log=lambda s: print(f"[instance] {s}", flush=True))
        md = timing_only_markdown(cfg, r, "python -m paper_2401_09670_amd.instance "
                                  + " ".join(argv if argv is not None else sys.argv[1:]))
        print(md)
        print(json.dumps(r, default=float))
        if a.out:
            with open(a.out, "w") as f:
                f.write(md)
        return 0
    n_req = a.requests or {3: 512, 4: 48, 5: 0}[a.config]
    reqs = requests_for(cfg, n_req)
    shape, L = cfg["shape"], cfg["layers"]
    weight_gb = L * 2.0 * (shape.hidden * shape.qkv_width + shape.hidden ** 2 + 2 * shape.hidden * shape.ffn) / 1e9
    pool_gb = a.pool_gb or max(8.0, min(160.0, 250.0 - weight_gb))
    plan = plan_for(cfg, reqs, pool_gb)

    def log(s):
        print(f"[instance] {s}", flush=True)

    log(f"{cfg['name']}: {len(reqs)} requests, weights {weight_gb:.1f} GB, pool {plan['pool_blocks']} pages "
        f"({plan['pool_blocks'] * plan['page_bytes'] / 1e9:.1f} GB)")
    stack = GpuStack(shape, L, cfg["seed"], plan["pool_blocks"], plan["max_batch"], plan["max_prefill_tokens"],
                     plan["max_ctx"], plan["max_blocks"], max_requests=len(reqs), overlap_handoff=a.overlap_handoff,
                     log=log)
    sched = Scheduler(reqs, BlockPool(plan["pool_blocks"], cfg["seed"]), plan["max_batch"], plan["token_cap"],
                      shape.block_size, plan["max_blocks"])
    raw = run_workload(stack, sched, a.max_steps or None, log)
    res = summarise(raw, shape, L)
    cmd = "python -m paper_2401_09670_amd.instance " + " ".join(argv if argv is not None else sys.argv[1:])
    md = to_markdown(cfg, plan, len(reqs), res, cmd)
    print(md)
    print(json.dumps({k: v for k, v in res.items()}, default=float))
    if a.out:
        with open(a.out, "w") as f:
            f.write(md)
    return 0


if __name__ == "__main__":
    sys.exit(main())
