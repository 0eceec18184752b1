"""ls_stage_decode_static, the entry point that allocates nothing: its K-split partial tiles
live in the library's static device array instead of the caller's workspace.  Same kernels,
same order, so its output must be bit-identical to ls_stage_decode's -- on two calls in a row,
the second with a smaller batch (the array keeps the first call's contents), and a step that
needs more than the array holds must be refused before anything is enqueued."""
import ctypes as C

import numpy as np
import pytest

import synth
from helpers import make_gpu, make_oracle, rel_l2, to_dev, to_host

pytestmark = pytest.mark.gpu

# 17..64 rows take the weight-streaming GEMMs that split K across workgroups
SHAPE = synth.StageShape("bf16", 2, 512, 8, 2, 64, 1408, 1000)


def test_static_scratch_decode_equals_workspace_decode_on_two_calls_the_second_smaller():
    import torch
    from paper_2502_09922_amd import LsError, binding as b

    seed, steps = 41, 2
    lengths = [int(n) for n in synth.ragged_lengths(seed, 48, 1, 20)]
    B, S, T = len(lengths), max(lengths), sum(lengths)
    twin = [make_gpu(SHAPE, seed, 0, 2, B, S + steps, T) for _ in range(2)]
    ora = make_oracle(SHAPE, seed, 0, 2, B, S + steps)
    tok = synth.token_ids(seed + 1, T, SHAPE.vocab)
    nt_o, _ = ora.prefill(tok, lengths)
    for st in twin:
        st.prefill(to_dev(SHAPE, tok), lengths)
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    # call 1: all 48 sequences; call 2: only the first 24 (their second new token)
    for step, batch in enumerate((B, B // 2)):
        feed = to_dev(SHAPE, nt_o[:batch].copy())
        ref_tok, ref_lg = twin[0].decode(feed, batch, S + step, want_logits=True)
        got_tok, got_lg = twin[1].decode(feed, batch, S + step, want_logits=True, static=True)
        torch.cuda.synchronize()
        assert torch.equal(got_lg, ref_lg), (step, batch)
        assert torch.equal(got_tok, ref_tok), (step, batch)
        assert torch.equal(twin[1].k, twin[0].k) and torch.equal(twin[1].v, twin[0].v)
        assert torch.equal(twin[1].seq_lens, twin[0].seq_lens)
        if step == 0:  # and both agree with the oracle (the same bar as every other parity test)
            nt_o, lg_o = ora.decode(nt_o)
            err = rel_l2(to_host(got_lg), lg_o)
            print("static decode vs oracle: rel-L2 %.3e" % err)
            assert err <= 2e-2
    # the logits tensors above come from torch; the library itself took no device memory
    assert torch.cuda.mem_get_info()[0] >= free_before - (64 << 20)
    for st in twin:
        st.close()


def test_static_scratch_decode_refuses_a_step_that_does_not_fit():
    import torch
    from paper_2502_09922_amd import LsError, binding as b

    # the 7B layer shape at 64 rows: the gate/up projection is cut into 4 K ranges across
    # workgroups, 4 x (gate + up) x 64 rows x 11008 columns x 4 bytes = 21.5 MiB: beyond 16 MiB
    big = synth.StageShape("bf16", 1, 4096, 32, 32, 128, 11008, 0)
    st = make_gpu(big, 3, 0, 1, 64, 8, 64)
    x = to_dev(big, synth.hidden_states(big, 4, 64))
    st.prefill(x, [1] * 64)
    st.seq_lens.fill_(-5)
    with pytest.raises(LsError) as e:
        st.decode(x, 64, 1, static=True)
    assert e.value.status == b.LS_ERR_OOM and "static" in str(e.value)
    torch.cuda.synchronize()
    assert (st.seq_lens.cpu() == -5).all()  # nothing was enqueued
    st.seq_lens.fill_(1)
    # 16 rows never split K across workgroups: no scratch needed, the call goes through
    a = st.decode(x[:16], 16, 1)
    st.seq_lens.fill_(1)
    c = st.decode(x[:16], 16, 1, static=True)
    torch.cuda.synchronize()
    assert torch.equal(a, c)
    st.close()
