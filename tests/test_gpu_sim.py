"""GPU: the simulator's decisions carried out on real page pools -- tick -> evict -> restore ->
append -> prefill / decode -- with every program's cache compared, bit for bit, with a record kept
outside the pools, and attention outputs compared with the oracle over that record; once with
bf16 caches and once with FP8 caches written by the quantising append."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_13692_amd import binding as ta
from paper_2602_13692_amd import sim_driver
from paper_2602_13692_amd import workloads as wl

import gpu_util as gu

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HQ, HKV, D, PS = 8, 2, 128, 16


class Record:
    """Every program's tokens (keys, values, queries), drawn once; what the caches must hold."""

    def __init__(self, n_programs, max_context, seed):
        gen = torch.Generator(device=DEV)
        gen.manual_seed(seed)
        self.k = torch.randn((n_programs, max_context, HKV, D), generator=gen, device=DEV).to(torch.bfloat16)
        self.v = torch.randn((n_programs, max_context, HKV, D), generator=gen, device=DEV).to(torch.bfloat16)
        self.q = torch.randn((n_programs, max_context, HQ, D), generator=gen, device=DEV).to(torch.bfloat16)

    def source(self, p, first, n):
        return self.k[p, first: first + n], self.v[p, first: first + n], self.q[p, first: first + n]

    def paged(self, p, c, which, scale=None):
        """[pages][Hkv][16][128] image of the program's first c tokens (zero padded): the bf16
        patterns as uint16, or with a scale the E4M3 codes the oracle's quantiser gives them."""
        pages = (c + PS - 1) // PS
        padded = torch.zeros((pages * PS, HKV, D), dtype=torch.bfloat16, device=DEV)
        padded[:c] = (self.k if which == "k" else self.v)[p, :c]
        paged = padded.view(pages, PS, HKV, D).permute(0, 2, 1, 3).contiguous()
        if scale is None:
            return wl.as_u16(paged)
        return oracle.quantise_e4m3(paged.float().cpu().numpy(), scale)


K_SCALE, V_SCALE = 0.021, 0.017      # N(0,1) values stay well inside +-448 code values


def _oracle_rows(rec, programs, q_lens, contexts, fp8=False):
    """The oracle's append-prefill over pools built from the record alone."""
    k_pages, v_pages, table, at = [], [], [], 0
    width = max((c + PS - 1) // PS for c in contexts)
    for p, c in zip(programs, contexts):
        kp, vp = rec.paged(p, c, "k", K_SCALE if fp8 else None), rec.paged(p, c, "v", V_SCALE if fp8 else None)
        row = np.full(width, -1, np.int32)
        row[: kp.shape[0]] = np.arange(at, at + kp.shape[0])
        at += kp.shape[0]
        k_pages.append(kp); v_pages.append(vp); table.append(row)
    q = torch.cat([rec.q[p, c - n: c] for p, n, c in zip(programs, q_lens, contexts)])
    cu = np.zeros(len(programs) + 1, np.int32)
    np.cumsum(q_lens, out=cu[1:])
    if fp8:
        return oracle.append_prefill_fp8(oracle.Geometry(HQ, HKV), wl.as_u16(q), cu, np.concatenate(k_pages),
                                         np.concatenate(v_pages), K_SCALE, V_SCALE, np.stack(table),
                                         np.array(contexts, np.int32))
    return oracle.append_prefill(oracle.Geometry(HQ, HKV), wl.as_u16(q), cu, np.concatenate(k_pages),
                                 np.concatenate(v_pages), np.stack(table), np.array(contexts, np.int32))


def _check_caches(rec, drv):
    """Active programs: their pool pages hold the record; paused ones: their host store does.
    (A program that has ended holds nothing any more.)  With an FP8 cache "the record" is the
    oracle's quantisation of it, and the comparison is as exact."""
    fp8 = drv.fp8
    elem = np.uint8 if fp8 else np.uint16
    as_elems = (lambda t: t.cpu().numpy()) if fp8 else wl.as_u16
    status = drv.sim.programs()["status"]
    for p in range(len(drv.context)):
        if int(status[p]) == ta.STATUS_TERMINATED:
            continue
        c = drv.context[p]
        pages = (c + PS - 1) // PS
        want_k = rec.paged(p, c, "k", K_SCALE if fp8 else None).reshape(pages, -1)
        want_v = rec.paged(p, c, "v", V_SCALE if fp8 else None).reshape(pages, -1)
        rows = c - (pages - 1) * PS                      # rows of the last page that exist
        if drv.table[p]:
            b = drv.backend[p]
            idx = torch.tensor(drv.table[p], device=DEV)
            got_k = as_elems(drv.k_pool[b].index_select(0, idx)).reshape(pages, -1)
            got_v = as_elems(drv.v_pool[b].index_select(0, idx)).reshape(pages, -1)
        else:
            got_k = drv.host_k[p][:pages].numpy().view(elem).reshape(pages, -1)
            got_v = drv.host_v[p][:pages].numpy().view(elem).reshape(pages, -1)
        # whole pages exactly; the last page on the rows that exist (the rest of a pool page may hold anything)
        assert np.array_equal(got_k[: pages - 1], want_k[: pages - 1]) and np.array_equal(got_v[: pages - 1], want_v[: pages - 1])
        last_got = got_k[pages - 1].reshape(HKV, PS, D)[:, :rows], got_v[pages - 1].reshape(HKV, PS, D)[:, :rows]
        last_want = want_k[pages - 1].reshape(HKV, PS, D)[:, :rows], want_v[pages - 1].reshape(HKV, PS, D)[:, :rows]
        assert np.array_equal(last_got[0], last_want[0]) and np.array_equal(last_got[1], last_want[1])
        assert drv.page_bytes == HKV * PS * D * (1 if fp8 else 2)


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16", "fp8"])
@pytest.mark.parametrize("n_backends,pool_pages,capacity", [(1, 170, 2500.0), (2, 95, 1400.0)])
def test_policy_drives_the_kernels_and_the_caches_stay_exact(n_backends, pool_pages, capacity, fp8):
    n, max_ctx = 10, 1400
    tr = wl.agent_trace(wl.SEED_BASE + 6000 + n_backends, n, n_turns=3, context_lo=150, context_hi=800, turn_lo=4,
                        turn_hi=20, tool_median_ticks=2.0, tool_sigma=1.0, out_lo=20, out_hi=150)
    sim = ta.Sim(n_backends, pool_pages, 4, max_ctx, 1.0, capacity, 1.0, 1.0, 2.0, tr.initial_context, tr.turn_tokens,
                 tr.tool_ticks, tr.tool_tokens)
    rec = Record(n, max_ctx, wl.SEED_BASE + 6100)
    fmt = dict(kv_format=ta.KV_FP8_E4M3, k_scale=K_SCALE, v_scale=V_SCALE) if fp8 else {}
    drv = sim_driver.Backends(sim, n_backends, pool_pages, HQ, HKV, max_ctx, tr.initial_context, rec.source, DEV, **fmt)
    checked_decodes = checked_prefills = 0
    for tick in range(400):
        drv.last_decode = drv.last_prefill = None
        drv.run_tick()
        torch.cuda.synchronize()
        if tick % 3 == 0:
            _check_caches(rec, drv)
        # attention results of the tick's last batches against the oracle over the record
        if drv.last_decode is not None and tick % 2 == 0:
            programs, out, lse = drv.last_decode
            ctx = [drv.context[p] for p in programs]
            ref, ref_lse = _oracle_rows(rec, programs, [1] * len(programs), ctx, fp8)
            gu.assert_close(out, lse, ref, ref_lse, f"decode, tick {tick}", lse_tol=gu.LSE_TOL_FP8 if fp8 else gu.LSE_TOL)
            checked_decodes += 1
        if drv.last_prefill is not None:
            programs, q_lens, out, lse = drv.last_prefill
            if all(len(drv.table[p]) > 0 for p in programs):       # still resident: contexts are the current ones
                ctx = [drv.context[p] for p in programs]
                # decode steps of the same tick have grown the contexts since: take them back
                # (a program decodes at most steps_per_tick tokens after its prefill)
                grown = {p: 0 for p in programs}
                for e in drv.sim_events:
                    if int(e["kind"]) == ta.SIM_DECODE and int(e["program"]) in grown:
                        grown[int(e["program"])] += 1
                ctx = [c - grown[p] for p, c in zip(programs, ctx)]
                ref, ref_lse = _oracle_rows(rec, programs, q_lens, ctx, fp8)
                gu.assert_close(out, lse, ref, ref_lse, f"prefill, tick {tick}", lse_tol=gu.LSE_TOL)
                checked_prefills += 1
        if all(int(s) == ta.STATUS_TERMINATED for s in sim.programs()["status"]):
            break
    else:
        pytest.fail("the trace did not finish")
    _check_caches(rec, drv)
    c = drv.counts
    assert checked_decodes > 5 and checked_prefills > 3
    assert c["restore"] >= n and c["release"] == n and c["decode_tokens"] > 0 and c["prefill_tokens"] > 0
    assert c["evict"] + c["evict_forced"] > 0, "the pools were sized so that programs have to make room"
    sim.close()
