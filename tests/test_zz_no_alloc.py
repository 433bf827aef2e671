"""-m gpu: dba_step_noalloc (the step with the library's own scratch, for callers that cannot allocate)
against dba_step_fmt, through the C ABI: same outputs, same state, same end of decoding, bit for bit,
on two decodes in a row that share the GPU's scratch array - the second one smaller, so that it runs
over what the first left behind - and on 16-bit log-probs; sizes beyond the array are refused."""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _decode_both_ways(torch, wl, fmt=None, mix=False):
    from paper_1804_06609_amd.session import Session
    toks, poff, soff = wl.csr()
    plain = Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff)
    own = Session(wl.B, wl.k, wl.V, wl.T, wl.eos_id, wl.pad_id, toks, poff, soff)
    tdt = {None: torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[fmt]
    for t in range(wl.T):
        lp = wl.logp(t)
        if fmt is None:
            dev = torch.from_numpy(lp).cuda()
        else:
            dev = torch.from_numpy(si.narrow16(lp, fmt).view(np.int16)).cuda().view(tdt)
        plain.step(dev)
        own.step(dev, noalloc=not (mix and t % 3 == 1))      # mix: every third step through the workspace
        for a, b, name in zip(plain.outputs(), own.outputs(), ("token", "backptr", "score", "flags")):
            assert a.tobytes() == b.tobytes(), (name, t)
        sa, sb = plain.state(), own.state()
        for name in sa:
            assert sa[name].tobytes() == sb[name].tobytes(), (name, t)
        assert plain.finished().tobytes() == own.finished().tobytes(), t
    for a, b in zip(plain.finalize(), own.finalize()):
        assert a.tobytes() == b.tobytes()
    plain.close()
    own.close()


def test_noalloc_step_matches_the_step_with_workspace_scratch():
    import torch
    assert torch.cuda.is_available()
    first = si.make_small(9801, 6, 33, 4099, 12, max_phrases=5, max_len=3, dup_prob=0.3)
    first.eos_switch = 6
    _decode_both_ways(torch, first)
    second = si.make_small(9802, 2, 5, 257, 9, max_phrases=3, max_len=2, dup_prob=0.3)   # smaller, right after
    second.eos_switch = 4
    _decode_both_ways(torch, second)
    third = si.make_small(9803, 3, 13, 1023, 8, max_phrases=4, max_len=3, dup_prob=0.3)
    third.eos_switch = 4
    _decode_both_ways(torch, third, fmt="bf16", mix=True)


def test_noalloc_step_at_the_headline_shape():
    import torch
    wl = si.make_config(4, T=6)
    _decode_both_ways(torch, wl)


def test_noalloc_step_refuses_more_rows_than_its_scratch_holds():
    import torch
    import paper_1804_06609_amd as dba
    from paper_1804_06609_amd.session import Session
    B, k, V = 129, 64, 64                                   # 8256 beam rows > DBA_NOALLOC_MAX_ROWS
    assert B * k > dba.DBA_NOALLOC_MAX_ROWS
    wl = si.make_small(9804, B, k, V, 2, max_phrases=1, max_len=1)
    toks, poff, soff = wl.csr()
    ses = Session(B, k, V, 2, wl.eos_id, wl.pad_id, toks, poff, soff)
    dev = torch.from_numpy(wl.logp(0)).cuda()
    with pytest.raises(dba.DbaError, match="DBA_NOALLOC_MAX_ROWS") as ei:
        ses.step(dev, noalloc=True)
    assert ei.value.code == dba.DBA_EINVAL and dba.dba_steps_done(ses.ctx) == 0
    ses.step(dev)                                           # the ordinary step still works
    assert dba.dba_steps_done(ses.ctx) == 1
    ses.close()


def test_noalloc_step_writes_only_inside_its_buffers():
    """The guard-band check of tests/test_gpu_robustness.py with every step taken through dba_step_noalloc."""
    from test_gpu_robustness import guarded_decode
    guarded_decode("noalloc")
