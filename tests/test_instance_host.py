"""Host-side bookkeeping of a serving instance (no GPU): page pool, first-come-first-served prefill
batches under a token cap, admission by free pages, the continuously refilled decode batch."""
import numpy as np
import pytest

from oracle import ds_oracle as orc
from paper_2401_09670_amd import instance as inst
from paper_2401_09670_amd import synth


def test_block_pool_hands_out_every_page_once():
    pool = inst.BlockPool(37, seed=3)
    a, b = pool.alloc(10), pool.alloc(27)
    assert pool.n_free == 0
    assert sorted(np.concatenate([a, b]).tolist()) == list(range(37))
    with pytest.raises(MemoryError):
        pool.alloc(1)
    pool.free(a)
    assert pool.n_free == 10
    assert sorted(pool.alloc(10).tolist()) == sorted(a.tolist())
    pool.free(b)
    with pytest.raises(RuntimeError):
        pool.free(np.arange(20))


def _simulate(reqs, num_blocks, max_batch, cap, check=True):
    """Drives the scheduler the way run_workload does, with no device: returns the admission order,
    the prefill batches, the number of decoding steps each request took part in and, per step, the
    batch size and whether requests were still queued behind it."""
    pool = inst.BlockPool(num_blocks, seed=1)
    sched = inst.Scheduler(reqs, pool, max_batch, cap)
    by_id = {r.rid: r for r in reqs}
    admitted, batches, steps, sizes = [], [], {r.rid: 0 for r in reqs}, []
    placed_order = []
    guard = 0
    while not sched.done:
        guard += 1
        assert guard < 100000
        progressed = True
        while progressed:
            n_done = len(sched.finished)
            placed = sched.place_ready()
            placed_order += [rid for _, rid in placed]
            batch = sched.next_prefill_batch()
            if batch:
                admitted += [s.req.rid for s in batch]
                batches.append([s.req.rid for s in batch])
                table = sched.prefill_table(batch)
                for i, s in enumerate(batch):
                    need = synth.blocks_needed(s.req.prompt_len, 16)
                    assert (table[i, :need] >= 0).all() and (table[i, need:] == -1).all()
            progressed = bool(placed) or bool(batch) or len(sched.finished) != n_done
        rows = sched.decode_rows()
        if not rows:
            assert not sched.waiting and not sched.ready
            break
        assert len(rows) <= max_batch
        sizes.append((len(rows), bool(sched.waiting or sched.ready)))
        ctx, table = sched.prepare_step(rows)
        if check:
            owned = [b for s in sched.ready for b in s.blocks]
            for i, row in enumerate(rows):
                s = sched.active[row]
                assert ctx[i] == s.ctx_len
                need = synth.blocks_needed(int(ctx[i]) + 1, 16)          # the new token's slot exists
                assert len(s.blocks) == need
                assert (table[i, :need] == s.blocks).all() and (table[i, need:] == -1).all()
                owned += s.blocks
            assert len(set(owned)) == len(owned)                          # no page shared
            assert pool.n_free + len(owned) == num_blocks                 # none lost
            promised = sum(s.reserved for s in list(sched.active.values()) + list(sched.ready))
            assert pool.n_free >= promised                                # reservations are backed by pages
        for row in rows:
            steps[sched.active[row].req.rid] += 1
        sched.finish_step(rows)
        sched.retire_finished()
    assert pool.n_free == num_blocks
    assert sorted(sched.finished) == sorted(by_id)
    multi = [r.rid for r in reqs if r.output_len > 1]
    assert placed_order == [rid for rid in admitted if rid in set(multi)]   # rows are given in arrival order
    return admitted, batches, steps, sizes


def test_every_request_is_served_in_order_and_decodes_output_minus_one_steps():
    cfg = synth.config(2)
    reqs = inst.requests_for(cfg, 200)
    plan = inst.plan_for(cfg, reqs, pool_gb=160.0)        # room for everything: only the cap and the rows limit
    admitted, batches, steps, sizes = _simulate(reqs, plan["pool_blocks"], 128, plan["token_cap"])
    assert admitted == sorted(admitted)                       # first come first served, nobody skipped
    for r in reqs:
        assert steps[r.rid] == r.output_len - 1               # the first token comes from the prefill pass
    by_id = {r.rid: r for r in reqs}
    toks = [sum(by_id[i].prompt_len for i in b) for b in batches]
    assert all(t <= plan["token_cap"] or len(b) == 1 for t, b in zip(toks, batches))
    # the prefill side works ahead of the decode rows, so its batches fill up to the cap: every batch but the
    # last stopped because the next prompt would not fit any more
    nxt = [by_id[b[-1] + 1].prompt_len for b in batches[:-1]]
    assert all(t + n > plan["token_cap"] for t, n in zip(toks[:-1], nxt))
    # and the decode batch stays full while requests are left to refill it
    assert all(n == 128 for n, more_to_come in sizes if more_to_come)
    assert any(more_to_come for _, more_to_come in sizes)


def test_small_pool_throttles_admission_but_nothing_starves():
    rng = np.random.default_rng(5)
    reqs = [inst.Request(i, int(rng.integers(1, 400)), int(rng.integers(1, 120))) for i in range(150)]
    biggest = max(synth.blocks_needed(r.prompt_len + r.output_len - 1, 16) for r in reqs)
    admitted, batches, steps, sizes = _simulate(reqs, biggest + 5, 16, 512)
    assert admitted == list(range(150))
    assert all(steps[r.rid] == r.output_len - 1 for r in reqs)


def test_request_that_can_never_fit_is_refused_up_front():
    with pytest.raises(ValueError):
        inst.Scheduler([inst.Request(0, 1000, 10)], inst.BlockPool(8), 4, 4096)


def test_single_token_requests_never_enter_the_decode_batch():
    reqs = [inst.Request(i, 20, 1) for i in range(10)]
    admitted, batches, steps, sizes = _simulate(reqs, 64, 4, 4096)
    assert admitted == list(range(10)) and all(v == 0 for v in steps.values())


def test_stage_workload_has_prefill_only_prompts_then_a_preloaded_decode_batch():
    cfg = synth.config(4)
    reqs = inst.requests_for(cfg, 0)
    assert [r.prompt_len for r in reqs[:8]] == [2048] * 8 and all(r.output_len == 1 for r in reqs[:8])
    pre = reqs[8:]
    assert len(pre) == 256 and all(r.preloaded and r.output_len == 33 for r in pre)
    assert all(128 <= r.prompt_len <= 2048 for r in pre)
    plan = inst.plan_for(cfg, reqs, pool_gb=160.0)
    admitted, batches, steps, sizes = _simulate(reqs, plan["pool_blocks"], plan["max_batch"], plan["token_cap"], check=False)
    assert batches[0] == list(range(8))                       # the 8 x 2048 prompts form one batch
    assert all(steps[r.rid] == 32 for r in pre)


def test_work_counts_match_the_formulas_of_the_latency_appendix():
    shape = synth.OPT_13B
    lens = [512, 300, 77]
    t = sum(lens)
    want = orc.prefill_gemm_flops(t, shape.hidden, shape.ffn) + orc.prefill_attention_flops(lens, shape.hidden)
    assert inst.prefill_flops(lens, shape, 1, vocab=0) == pytest.approx(want, rel=1e-12)
    assert inst.prefill_flops(lens, shape, 5, vocab=0) == pytest.approx(5 * want, rel=1e-12)
    ctx = [511, 20, 4000, 9]
    B = len(ctx)
    want_b = 2 * (orc.decode_gemm_traffic_elems(B, shape.hidden, shape.ffn)
                  + orc.decode_attention_kv_elems(ctx, shape.hidden))
    got = inst.decode_bytes(ctx, shape, 1, vocab=0)
    # the appendix's GEMM count omits what attention itself reads and writes besides K and V
    # (q in, o out: 2 B h elements) and the appended K/V rows (2 B h): 8 B h bytes in all
    assert got == pytest.approx(want_b, abs=8 * B * shape.hidden + 1)
