"""2D pipelined execution (Section 4.3, Fig. 6a): several stages on their own streams, several
micro-batches in flight.  What is unique is checked exactly: every micro-batch's result must
be bit-identical to the same stage handles run one call after the other on one stream (the
kernels and their order per micro-batch are the same; only the interleaving differs), and it
must match the CPU oracle within the benchmark tolerance."""
import numpy as np
import pytest

import synth
from helpers import check_close, greedy_agreement, make_gpu, make_oracle, packed_blocks, rel_l2, to_dev, to_host

pytestmark = pytest.mark.gpu

SHAPE = synth.StageShape("bf16", 4, 512, 8, 2, 64, 1408, 1000)
SEED = 31


def serial_reference(stages, mb_kv, inputs, lengths, dec_inputs):
    """Each micro-batch through the stages, one call after the other on the null stream."""
    import ctypes as C
    import torch
    from paper_2502_09922_amd import binding as b

    outs = []
    for m, (x, lens) in enumerate(zip(inputs, lengths)):
        per = []
        cur = x
        for s, st in enumerate(stages):
            st.kv = mb_kv[m][s]  # this micro-batch's cache in this stage
            cur = st.prefill(cur, lens)
        per.append(cur.clone())
        for t, xs in enumerate(dec_inputs[m]):
            cur = xs
            for s, st in enumerate(stages):
                st.kv = mb_kv[m][s]
                cur = st.decode(cur, len(lens), max(lens) + t)
            per.append(cur.clone())
        torch.cuda.synchronize()
        outs.append(per)
    return outs


@pytest.mark.parametrize("cuts", [(0, 2, 4), (0, 1, 3, 4)])
def test_pipelined_microbatches_equal_serial_runs_and_the_oracle(cuts):
    import torch
    from paper_2502_09922_amd import MicroBatch, Pipeline

    lengths = [[33, 8, 70], [64], [5, 5, 129, 17]]
    steps = 3
    max_b = max(len(l) for l in lengths)
    max_s = max(max(l) for l in lengths) + steps
    max_t = max(sum(l) for l in lengths)
    spans = list(zip(cuts[:-1], cuts[1:]))
    stages = [make_gpu(SHAPE, SEED, lo, hi, max_b, max_s, max_t) for lo, hi in spans]
    first_tok = stages[0].first
    pipe = Pipeline(stages)
    mbs = [MicroBatch(pipe, max_t) for _ in lengths]

    def gen_in(seed, rows):
        return to_dev(SHAPE, synth.token_ids(seed, rows, SHAPE.vocab) if first_tok
                      else synth.hidden_states(SHAPE, seed, rows))

    inputs = [gen_in(SEED + 1 + m, sum(l)) for m, l in enumerate(lengths)]
    # pipelined: prompt pass of all micro-batches, then `steps` generation steps; the model
    # has an LM head, so each step feeds the tokens the previous call produced
    o, lg = pipe.run(0, mbs, inputs, lengths=lengths, want_logits=True)
    toks, logits = [o], [lg]
    for t in range(steps):
        o, lg = pipe.run(1, mbs, toks[-1], max_ctx=[max(l) + t for l in lengths], want_logits=True)
        toks.append(o)
        logits.append(lg)
    torch.cuda.synchronize()
    got = [[toks[t][m].clone() for t in range(steps + 1)] for m in range(len(lengths))]
    got_k = [[c[0].clone() for c in mb.caches] for mb in mbs]

    # serial reference on fresh caches, fed with the same token sequence
    ref_mbs = [MicroBatch(pipe, max_t) for _ in lengths]
    ref = serial_reference(stages, [[mb.kv[s] for s in range(len(stages))] for mb in ref_mbs], inputs, lengths,
                           [[got[m][t] for t in range(steps)] for m in range(len(lengths))])
    for m in range(len(lengths)):
        for t in range(steps + 1):
            assert torch.equal(got[m][t], ref[m][t]), (m, t)
        for s in range(len(stages)):
            assert torch.equal(got_k[m][s], ref_mbs[m].caches[s][0]), (m, s)

    # and against the oracle: whole model, teacher-forced with the pipeline's own tokens
    for m, lens in enumerate(lengths):
        ora = make_oracle(SHAPE, SEED, 0, SHAPE.n_layers_total, len(lens), max_s)
        nt, lg = ora.prefill(synth.token_ids(SEED + 1 + m, sum(lens), SHAPE.vocab), lens)
        adj = n = 0
        for t in range(steps + 1):
            mine = got[m][t].cpu().numpy()
            lg_g = to_host(logits[t][m])
            check_close(lg_g, lg, "bf16", "pipelined micro-batch %d call %d" % (m, t))
            _, a_, n_ = greedy_agreement(mine, lg_g, nt, lg)
            adj += a_
            n += n_
            if t < steps:
                nt, lg = ora.decode(mine.astype(np.int32))
        assert adj >= 0.99 * n, (m, adj, n)
    pipe.close()
    for st in stages:
        st.close()


def test_pipeline_rejects_stages_that_do_not_follow_each_other():
    import ctypes as C
    from paper_2502_09922_amd import LsError, Pipeline, binding as b

    a = make_gpu(SHAPE, SEED, 0, 2, 2, 16, 16, load=False)
    c = make_gpu(SHAPE, SEED, 3, 4, 2, 16, 16, load=False)
    with pytest.raises(LsError) as e:
        Pipeline([a, c])
    assert e.value.status == b.LS_ERR_INVALID_ARG
    other = make_gpu(SHAPE.with_(ffn=704), SEED, 2, 4, 2, 16, 16, load=False)
    with pytest.raises(LsError):
        Pipeline([a, other])
    a.close(); c.close(); other.close()


def test_a_failing_pipeline_pass_enqueues_nothing_in_any_stage():
    """Errors that only a later stage or a later micro-batch shows (a block never enqueued for
    load, a malformed cu_seqlens) are found before the first enqueue: no stage's cache
    lengths move."""
    import ctypes as C
    import torch
    from paper_2502_09922_amd import LsError, MicroBatch, Pipeline, binding as b

    a = make_gpu(SHAPE, SEED, 0, 2, 2, 32, 32)
    c = make_gpu(SHAPE, SEED, 2, 4, 2, 32, 32, load=False)  # holds layers 2, 3 and the head: none loaded
    pipe = Pipeline([a, c])
    mbs = [MicroBatch(pipe, 32) for _ in range(2)]
    for mb in mbs:
        for _, _, sl in mb.caches:
            sl.fill_(-3)
    x = [to_dev(SHAPE, synth.token_ids(SEED + m, 12, SHAPE.vocab)) for m in range(2)]
    with pytest.raises(LsError) as e:
        pipe.run(0, mbs, x, lengths=[[5, 7], [12]])
    assert e.value.status == b.LS_ERR_NOT_LOADED
    blocks = packed_blocks(c, SEED)
    for l, buf in blocks.items():
        c.load_block(l, c.stage_host_block(l, buf))
    # micro-batch 1 declares 12 rows but its cu_seqlens ends at 11
    arr = (b.ls_microbatch * 2)()
    keep = []
    for m, lens in enumerate([[5, 7], [11]]):
        cu = np.zeros(len(lens) + 1, np.int32)
        cu[1:] = np.cumsum(lens)
        cu_dev = torch.from_numpy(cu).cuda()
        out = torch.empty(len(lens), dtype=torch.int32, device="cuda")
        keep += [cu, cu_dev, out]
        arr[m].in_ = x[m].data_ptr()
        arr[m].cu_seqlens_dev = cu_dev.data_ptr()
        arr[m].cu_seqlens_host = cu.ctypes.data_as(C.POINTER(C.c_int32))
        arr[m].batch, arr[m].total_tokens = len(lens), 12
        arr[m].kv, arr[m].handoff, arr[m].out = mbs[m].kv, mbs[m].handoff, out.data_ptr()
    torch.cuda.synchronize()
    assert b.ls_pipeline_run(pipe.handle, 0, arr, 2, pipe._stream_ptrs) == b.LS_ERR_INVALID_ARG
    torch.cuda.synchronize()
    for mb in mbs:
        for _, _, sl in mb.caches:
            assert (sl.cpu() == -3).all()
    # the same pipeline still runs a well-formed pass
    pipe.run(0, mbs, x, lengths=[[5, 7], [12]])
    torch.cuda.synchronize()
    assert mbs[0].caches[1][2].cpu().tolist() == [5, 7] and mbs[1].caches[0][2].cpu().tolist()[:1] == [12]
    pipe.close(); a.close(); c.close()
