"""-m gpu: checks of the device side that compare the HIP path with itself or with guard patterns
rather than with the oracle: the same decode twice gives the same bytes, and a decode writes nowhere
outside the buffers it was given."""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _decode(torch, wl, options=None, fmt=None):
    """All bytes a decode leaves behind: every step's outputs, state and stopping bits, and the
    end of decoding (which walks the recorded history)."""
    from paper_1804_06609_amd.session import Session
    toks, poff, soff = wl.csr()
    ses = Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff, options=options)
    trace = []
    for t in range(wl.T):
        lp = wl.logp(t)
        if fmt is None:
            dev = torch.from_numpy(lp).cuda()
        else:
            dev = torch.from_numpy(si.narrow16(lp, fmt).view(np.int16)).cuda().view(torch.bfloat16)
        ses.step(dev)
        trace.extend(a.tobytes() for a in ses.outputs())
        st = ses.state()
        trace.extend(st[name].tobytes() for name in sorted(st))
        trace.append(ses.finished().tobytes())
    trace.extend(np.asarray(a).tobytes() for a in ses.finalize())
    ses.close()
    return trace


@pytest.mark.parametrize("paper_setup", [False, True])
def test_the_same_decode_twice_gives_the_same_bytes(paper_setup):
    """Config-3 shapes (16 sentences, k = 10, V = 32000; boosted constraint tokens, so phrases start
    and break), 40 steps with end-of-sentence from step 25, bare and with the options of Sec. 4 on."""
    import torch
    from paper_1804_06609_amd import DBA_OPT_NORMALIZE_FINISHED, DBA_OPT_PRUNE_THRESHOLD, DBA_OPT_TRACK_COMPLETED
    wl = si.make_config(3, T=40)
    wl.eos_switch = 25
    opts = {DBA_OPT_NORMALIZE_FINISHED: 1, DBA_OPT_PRUNE_THRESHOLD: 20.0, DBA_OPT_TRACK_COMPLETED: 1} if paper_setup else None
    first = _decode(torch, wl, opts)
    second = _decode(torch, wl, opts)
    assert first == second


def test_the_same_bf16_decode_twice_gives_the_same_bytes():
    import torch
    wl = si.make_small(9951, 5, 20, 12345, 14, max_phrases=5, max_len=3, dup_prob=0.3)
    wl.eos_switch = 7
    assert _decode(torch, wl, fmt="bf16") == _decode(torch, wl, fmt="bf16")


GUARD = 1 << 16           # bytes of guard band on each side
PATTERN = 0xA5


class _Guarded:
    """A device buffer of `nbytes` with a guard band before and after it, filled with a pattern."""

    def __init__(self, torch, nbytes, align=256):
        self.torch = torch
        self.raw = torch.full((nbytes + 2 * GUARD + align,), PATTERN, dtype=torch.uint8, device="cuda")
        start = (self.raw.data_ptr() + GUARD + align - 1) // align * align
        self.off = start - self.raw.data_ptr()
        self.ptr, self.nbytes = start, nbytes

    def body(self):
        return self.raw[self.off:self.off + self.nbytes]

    def guards_intact(self):
        lo = self.raw[:self.off]
        hi = self.raw[self.off + self.nbytes:]
        return bool((lo == PATTERN).all().item()) and bool((hi == PATTERN).all().item())


@pytest.mark.parametrize("case", ["k64_c64", "odd_v", "bf16_odd_v"])
def test_a_decode_writes_only_inside_its_buffers(case):
    guarded_decode(case)


def guarded_decode(case):
    """Workspace and the four output arrays sit between guard bands; after decodes with the widest beam
    and the most constraint tokens (k = 64, 64 tokens), with rows of odd length (unaligned rows, ragged
    tiles) in fp32 and bf16, bare and with the options of Sec. 4 on, every guard byte is
    as it was, and the outputs agree with an unguarded run."""
    import torch
    import paper_1804_06609_amd as dba
    if case == "k64_c64":
        B, k, V, T = 3, 64, 5003, 8
        cons = si.fixed_total_constraints(61, B, V, 64, max_len=4)
        wl = si.Workload(B=B, k=k, V=V, T=T, seed=61, constraints=cons,
                         boost_tokens=[[w for p in s for w in p] for s in cons], boost_prob=0.3, boost_value=6.0)
    else:
        wl = si.make_small(9961, 4, 13, 4099, 10, max_phrases=5, max_len=3, dup_prob=0.3)
    wl.eos_switch = wl.T // 2
    fmt = "bf16" if case == "bf16_odd_v" else None
    want = _decode(torch, wl, fmt=fmt)
    toks, poff, soff = wl.csr()
    B, k, V, T = wl.B, wl.k, wl.V, wl.T
    stream = torch.cuda.current_stream()
    for options in ({}, {dba.DBA_OPT_NORMALIZE_FINISHED: 1, dba.DBA_OPT_PRUNE_THRESHOLD: 20.0,
                         dba.DBA_OPT_TRACK_COMPLETED: 1}):
        ws = _Guarded(torch, dba.dba_workspace_bytes(B, k, V, T, dba.DBA_MAX_CONS_TOKENS))
        o_tok, o_bp, o_sc = (_Guarded(torch, B * k * 4, align=4) for _ in range(3))
        o_fl = _Guarded(torch, B * k, align=1)
        ctx = dba.dba_init(B, k, V, T, wl.eos_id, wl.pad_id, toks, poff, soff, ws.ptr, ws.nbytes, stream.cuda_stream)
        for opt, val in options.items():
            dba.dba_set_option(ctx, opt, val)
        got = []
        for t in range(T):
            lp = wl.logp(t)
            if fmt is None:
                dev = torch.from_numpy(lp).cuda()
                code = dba.DBA_LOGP_F32
            else:
                dev = torch.from_numpy(si.narrow16(lp, fmt).view(np.int16)).cuda().view(torch.bfloat16)
                code = dba.DBA_LOGP_BF16
            step = dba.dba_step_noalloc if case == "noalloc" else dba.dba_step_fmt
            step(ctx, dev.data_ptr(), code, o_tok.ptr, o_bp.ptr, o_sc.ptr, o_fl.ptr)
            torch.cuda.synchronize()
            got.append(o_tok.body().cpu().numpy().tobytes())
            got.append(o_bp.body().cpu().numpy().tobytes())
            got.append(o_sc.body().cpu().numpy().tobytes())
            got.append(o_fl.body().cpu().numpy().tobytes())
        fin = (np.empty((B, T), np.int32), np.empty(B, np.int32), np.empty(B, np.float32), np.empty(B, np.int32))
        dba.dba_finalize(ctx, *fin)
        dba.dba_destroy(ctx)
        for g in (ws, o_tok, o_bp, o_sc, o_fl):
            assert g.guards_intact(), (case, options)
        if not options:
            # the unguarded run's trace holds, per step, the four outputs first
            per_step = len(want[:-4]) // T
            for t in range(T):
                assert got[4 * t:4 * t + 4] == want[per_step * t:per_step * t + 4], (case, t)
            assert [a.tobytes() for a in fin] == want[-4:]


def test_a_decode_replayed_from_a_hip_graph_matches_eager_launches():
    """A step enqueues two kernels and nothing else (no allocation, no memset, no copy), so a decode can
    be recorded into a HIP graph by a caller who wants to.  Steps 1..T-1 of a decode are recorded once and replayed three times, each
    time from the device state after step 0 (the workspace is copied back, with eager work and
    synchronisations in between); every replay must leave the beam, the state and the end of
    decoding of the eager decode."""
    import torch
    from paper_1804_06609_amd.session import Session
    wl = si.make_config(3, T=24)
    wl.eos_switch = 14
    toks, poff, soff = wl.csr()
    dev = [torch.from_numpy(wl.logp(t)).cuda() for t in range(wl.T)]
    eager = Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff)
    for t in range(wl.T):
        eager.step(dev[t])
    want_out = [a.tobytes() for a in eager.outputs()]
    want_state = {n: a.tobytes() for n, a in eager.state().items()}
    want_fin = [np.asarray(a).tobytes() for a in eager.finalize()]
    want_stop = eager.finished().tobytes()
    eager.close()

    side = torch.cuda.Stream()
    ses = Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff, stream=side)
    with torch.cuda.stream(side):
        ses.step(dev[0])
    torch.cuda.synchronize()
    after_step0 = ses.workspace.clone()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for t in range(1, wl.T):
            ses.step(dev[t])
    torch.cuda.synchronize()
    for replay in range(3):
        ses.workspace.copy_(after_step0)                  # eager work between the replays
        for o in (ses.out_token, ses.out_backptr, ses.out_score, ses.out_flags):
            o.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            graph.replay()
        torch.cuda.synchronize()
        assert [a.tobytes() for a in ses.outputs()] == want_out, replay
        assert {n: a.tobytes() for n, a in ses.state().items()} == want_state, replay
        assert ses.finished().tobytes() == want_stop, replay
        assert [np.asarray(a).tobytes() for a in ses.finalize()] == want_fin, replay
    ses.close()
