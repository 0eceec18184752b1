"""Parity of the HIP stage (through the C ABI) with the CPU oracle on the same seeded bytes.

Tolerances are the benchmark definition's: relative L2 error <= 1e-4 (fp32 path) and
<= 2e-2 (bf16 path) on final hidden states / logits; greedy tokens are compared
teacher-forced, and a position whose oracle top-1/top-2 margin is below 4x the measured
max-abs logit error counts as a declared tie.
"""
import numpy as np
import pytest

import synth
from helpers import (TOL, check_close, check_delta, greedy_agreement, make_gpu, make_oracle, packed_blocks, rel_l2,
                     to_dev, to_host)

pytestmark = pytest.mark.gpu

# a small bf16 decoder with grouped-query attention, several tiles wide plus ragged tails
MINI_BF16 = synth.StageShape("bf16", 3, 512, 8, 2, 64, 1408, 1000)
MINI_BF16_HD128 = synth.StageShape("bf16", 2, 768, 6, 6, 128, 2080, 0)


def run_full_model(shape, seed, lengths, steps):
    """Whole model as one stage: prompt pass then teacher-forced greedy decode."""
    import torch

    B, S = len(lengths), max(lengths)
    gpu = make_gpu(shape, seed, 0, shape.n_layers_total, B, S + steps, sum(lengths))
    ora = make_oracle(shape, seed, 0, shape.n_layers_total, B, S + steps)
    tok = synth.token_ids(seed + 1, sum(lengths), shape.vocab)
    nt_o, lg_o = ora.prefill(tok, lengths)
    nt_g, lg_g = gpu.prefill(to_dev(shape, tok), lengths, want_logits=True)
    what = "%s d%d V%d B%d" % (shape.dtype, shape.hidden, shape.vocab, B)
    errs = [check_close(to_host(lg_g), lg_o, shape.dtype, what + " prompt logits")["rel_l2"]]
    agree = [greedy_agreement(nt_g.cpu().numpy(), to_host(lg_g), nt_o, lg_o, shape.dtype)]
    for t in range(steps):
        feed = nt_o.copy()  # teacher forcing: both sides consume the oracle's tokens
        nt_o, lg_o = ora.decode(feed)
        nt_g, lg_g = gpu.decode(to_dev(shape, feed), B, S + t, want_logits=True)
        errs.append(check_close(to_host(lg_g), lg_o, shape.dtype, what + " step %d logits" % t)["rel_l2"])
        agree.append(greedy_agreement(nt_g.cpu().numpy(), to_host(lg_g), nt_o, lg_o, shape.dtype))
    assert gpu.seq_lens.cpu().numpy()[:B].tolist() == [n + steps for n in lengths]
    gpu.close()
    return errs, agree


def test_tiny_fp32_whole_model_prefill_and_decode():
    """Benchmark config 1: 2 layers, d=256, 4x64 heads, F=688, V=512; prompt 32, 8 steps."""
    errs, agree = run_full_model(synth.CONFIGS["tiny_f32"], 0, [32], 8)
    assert max(errs) <= TOL["f32"], errs
    assert all(raw == n for raw, _, n in agree), agree


def test_mini_bf16_ragged_whole_model():
    errs, agree = run_full_model(MINI_BF16, 11, [17, 64, 1, 33, 128, 5], 6)
    assert max(errs) <= TOL["bf16"], errs
    raw = sum(a[0] for a in agree)
    adj = sum(a[1] for a in agree)
    n = sum(a[2] for a in agree)
    assert adj >= 0.99 * n, (raw, adj, n)


@pytest.mark.parametrize("shape,lengths", [
    (MINI_BF16.with_(vocab=0), [70, 3, 129]),
    (MINI_BF16_HD128, [131, 64, 9]),
    # grouped-query heads of 128: the matrix-core decode attention (3 and 8 heads per kv head),
    # contexts from under one 32-key tile to several tiles per wavefront
    (MINI_BF16_HD128.with_(n_kv_heads=2), [131, 64, 9, 1, 31, 32, 33]),
    (MINI_BF16_HD128.with_(hidden=1024, n_q_heads=8, n_kv_heads=1), [300, 2, 257]),
    (synth.CONFIGS["tiny_f32"].with_(vocab=0), [5, 40, 13]),
])
def test_middle_stage_hidden_parity_and_decode(shape, lengths):
    seed, steps, B = 21, 5, len(lengths)
    S = max(lengths)
    lo, hi = 0, shape.n_layers_total
    gpu = make_gpu(shape, seed, lo, hi, B, S + steps, sum(lengths))
    ora = make_oracle(shape, seed, lo, hi, B, S + steps)
    x = synth.hidden_states(shape, seed + 1, sum(lengths))
    want = ora.prefill(x, lengths)
    got = to_host(gpu.prefill(to_dev(shape, x), lengths))
    what = "%s d%d Hq%d/Hkv%d hd%d" % (shape.dtype, shape.hidden, shape.n_q_heads, shape.n_kv_heads, shape.head_dim)
    # whole output, every row (a bad ragged tail), every column (a bad tile edge), every element
    check_close(got, want, shape.dtype, what + " prompt")
    from oracle.stage_oracle import decode_values
    check_delta(got, want, decode_values(x), shape.dtype, what + " prompt")
    for t in range(steps):
        xs = synth.hidden_states(shape, seed + 2 + t, B)
        want = ora.decode(xs)
        got = to_host(gpu.decode(to_dev(shape, xs), B, S + t))
        check_close(got, want, shape.dtype, what + " step %d" % t)
        check_delta(got, want, decode_values(xs), shape.dtype, what + " step %d" % t)
    gpu.close()


def test_grouped_query_decode_with_contexts_of_128_and_2048_in_one_batch():
    """Decode attention of a grouped-query model cuts contexts beyond 512 keys into chunks that
    run as workgroups of their own and are merged in a second pass: short and long contexts in
    one batch, lengths on both sides of the chunk and tile edges, several steps."""
    shape = synth.StageShape("bf16", 2, 512, 8, 2, 128, 704, 0)
    seed, steps = 47, 3
    lengths = [128, 2048, 511, 512, 513, 1024, 1025, 31, 1535]
    B, S = len(lengths), max(lengths)
    gpu = make_gpu(shape, seed, 0, 2, B, S + steps + 1, sum(lengths))
    ora = make_oracle(shape, seed, 0, 2, B, S + steps + 1)
    x = synth.hidden_states(shape, seed + 1, sum(lengths))
    check_close(to_host(gpu.prefill(to_dev(shape, x), lengths)), ora.prefill(x, lengths), "bf16", "GQA ragged prompt")
    for t in range(steps):
        xs = synth.hidden_states(shape, seed + 2 + t, B)
        check_close(to_host(gpu.decode(to_dev(shape, xs), B, S + t)), ora.decode(xs), "bf16", "GQA ragged step %d" % t)
    # a caller that understates the longest context still gets every key attended to
    xs = synth.hidden_states(shape, seed + 9, B)
    want = ora.decode(xs)
    check_close(to_host(gpu.decode(to_dev(shape, xs), B, 600)), want, "bf16", "GQA ragged step, max_ctx understated")
    gpu.close()


def test_prompt_gemm_edges_rows_and_columns_that_fill_no_whole_tile_or_vector():
    """The prompt GEMM stores four consecutive columns per lane and works on 256 x 256 tiles:
    a FFN width that is no multiple of four (the gate-up GEMM then takes its element-wise
    store path, the down projection a K that is no multiple of 64), prompt rows that end inside
    a tile, widths that end inside a 16-column MFMA tile."""
    for ffn, d, lengths in ((690, 256, [70, 33, 1]), (1412, 384, [131, 200]), (700, 320, [257])):
        shape = synth.StageShape("bf16", 2, d, d // 64, d // 64, 64, ffn, 0)
        seed = 61
        B, S = len(lengths), max(lengths)
        gpu = make_gpu(shape, seed, 0, 2, B, S + 2, sum(lengths))
        ora = make_oracle(shape, seed, 0, 2, B, S + 2)
        x = synth.hidden_states(shape, seed + 1, sum(lengths))
        tag = "d%d F%d T%d" % (d, ffn, sum(lengths))
        check_close(to_host(gpu.prefill(to_dev(shape, x), lengths)), ora.prefill(x, lengths), "bf16", tag + " prompt")
        xs = synth.hidden_states(shape, seed + 2, B)
        check_close(to_host(gpu.decode(to_dev(shape, xs), B, S)), ora.decode(xs), "bf16", tag + " step")
        gpu.close()


def test_prompt_gemm_workgroups_that_walk_several_tiles():
    """The prompt GEMM runs 256 workgroups that each walk tiles l, l + 256, ... as one stream of
    k-steps, the fills of a tile's last two k-steps already fetching the next tile: prompt
    passes whose gate-up GEMM has more than 256 tiles, with ragged last tile rows and columns,
    with an odd number of k-steps per tile (the LDS stage a tile starts in then alternates
    from tile to tile) and an even one."""
    for ffn, d, lengths in ((1412, 320, [2047, 2300, 2654, 2000]), (1800, 256, [3000, 2999, 1300])):
        shape = synth.StageShape("bf16", 2, d, d // 64, d // 64, 64, ffn, 0)
        seed = 67
        B, S = len(lengths), max(lengths)
        T = sum(lengths)
        assert ((T + 255) // 256) * ((ffn + 127) // 128) > 256 and T % 256 and ffn % 128
        gpu = make_gpu(shape, seed, 0, 2, B, S + 2, T)
        ora = make_oracle(shape, seed, 0, 2, B, S + 2)
        x = synth.hidden_states(shape, seed + 1, T)
        tag = "d%d F%d T%d" % (d, ffn, T)
        check_close(to_host(gpu.prefill(to_dev(shape, x), lengths)), ora.prefill(x, lengths), "bf16", tag + " prompt")
        xs = synth.hidden_states(shape, seed + 2, B)
        check_close(to_host(gpu.decode(to_dev(shape, xs), B, S)), ora.decode(xs), "bf16", tag + " step")
        gpu.close()


@pytest.mark.parametrize("shape,n_seq", [(MINI_BF16, 70), (MINI_BF16_HD128.with_(vocab=1000), 130)])
def test_more_than_64_sequences(shape, n_seq):
    """Beyond 64 rows a decode step leaves the weight-streaming GEMMs for the prompt pass's MFMA
    GEMM (one ragged tile row), the rotation kernel runs on its own, and the LM head of both
    passes is the MFMA GEMM's fp32 store."""
    rng = np.random.default_rng(83)
    lengths = [int(n) for n in rng.integers(1, 13, size=n_seq)]
    errs, agree = run_full_model(shape, 83, lengths, 3)
    assert max(errs) <= TOL["bf16"], errs
    adj = sum(a[1] for a in agree)
    n = sum(a[2] for a in agree)
    assert adj >= 0.99 * n, agree


def test_split_stages_equal_whole_stage():
    """Running layers [0,k) then [k,L) as two stages equals one stage [0,L)."""
    shape, seed, lengths = MINI_BF16.with_(vocab=0), 5, [33, 8]
    B, S = len(lengths), max(lengths)
    x = synth.hidden_states(shape, seed + 1, sum(lengths))
    whole = make_gpu(shape, seed, 0, 3, B, S + 2, sum(lengths))
    ref = whole.prefill(to_dev(shape, x), lengths)
    xs = synth.hidden_states(shape, seed + 2, B)
    ref_d = whole.decode(to_dev(shape, xs), B, S)
    ora = make_oracle(shape, seed, 0, 3, B, S + 2)
    want = ora.prefill(x, lengths)
    for k in (1, 2):
        a = make_gpu(shape, seed, 0, k, B, S + 2, sum(lengths))
        b = make_gpu(shape, seed, k, 3, B, S + 2, sum(lengths))
        got = b.prefill(a.prefill(to_dev(shape, x), lengths), lengths)
        got_d = b.decode(a.decode(to_dev(shape, xs), B, S), B, S)
        # Inside a stage the residual stream is fp32; the hand-off rounds it to bf16 once (at
        # most 2^-9 per element, about 0.3 * 2^-8 in relative L2), and where that moves the
        # second stage's result across a rounding boundary of its own bf16 output the two
        # outputs differ by one more such step: at most 2^-8 in relative L2, not bitwise.
        e_p, e_d = rel_l2(to_host(got), to_host(ref)), rel_l2(to_host(got_d), to_host(ref_d))
        print("split at %d: two stages vs one, rel-L2 %.2e (prompt) %.2e (step); 2^-8 = %.2e" % (k, e_p, e_d, 2.0**-8))
        assert e_p <= 2.0**-8 and e_d <= 2.0**-8
        check_close(to_host(got), want, "bf16", "two stages split at %d vs oracle" % k)
        a.close(); b.close()
    whole.close()


def test_streamed_equals_preloaded_bitwise_any_arrival_order_and_no_early_reads():
    """Blocks copied on a side stream while prefill runs give bit-identical results to a
    preloaded stage, in layer order and in the circularly shifted order of Algorithm 1
    (second half of the blocks first); a NaN-poisoned slab shows no kernel reads a block
    before its gate."""
    import torch

    shape, seed, lengths = MINI_BF16, 9, [40, 7, 90]
    B, S = len(lengths), max(lengths)
    tok = to_dev(shape, synth.token_ids(seed + 1, sum(lengths), shape.vocab))
    pre = make_gpu(shape, seed, 0, 3, B, S + 1, sum(lengths))
    torch.cuda.synchronize()
    ref_tok, ref_lg = pre.prefill(tok, lengths, want_logits=True)
    ref_k = pre.k.clone()
    import ctypes as C
    from paper_2502_09922_amd import binding as b

    ids = [-1, 0, 1, 2, 3]
    orders = []
    for group in (0, 1):  # the orders Algorithm 1 gives two sub-groups for these 5 blocks
        arr = (C.c_int32 * len(ids))()
        assert b.ls_plan_kway_order(len(ids), 2, group, arr) == 0
        orders.append([ids[i] for i in arr])
    assert orders == [[-1, 0, 1, 2, 3], [2, 3, -1, 0, 1]]
    for order in orders:
        st = make_gpu(shape, seed, 0, 3, B, S + 1, sum(lengths), load=False)
        st.slab.view(torch.int16).fill_(0x7FC0)  # bf16 NaN everywhere
        blocks = {l: st.stage_host_block(l, buf) for l, buf in packed_blocks(st, seed).items()}
        copy_stream = torch.cuda.Stream()
        torch.cuda.synchronize()
        for l in order:
            st.load_block(l, blocks[l], stream=copy_stream)
        got_tok, got_lg = st.prefill(tok, lengths, want_logits=True)
        torch.cuda.synchronize()
        assert torch.equal(got_lg, ref_lg) and torch.equal(got_tok, ref_tok)
        assert torch.equal(st.k, ref_k)
        assert not torch.isnan(got_lg).any()
        st.close()
    pre.close()


def test_runtime_errors_enqueue_nothing():
    import ctypes as C
    import torch
    from paper_2502_09922_amd import LsError, binding as b

    shape = synth.CONFIGS["tiny_f32"]
    st = make_gpu(shape, 0, 0, 2, 2, 16, 24, load=False)
    blocks = {l: st.stage_host_block(l, buf) for l, buf in packed_blocks(st, 0).items()}
    tok = to_dev(shape, synth.token_ids(1, 8, shape.vocab))
    st.seq_lens.fill_(-7)
    with pytest.raises(LsError) as e:
        st.prefill(tok, [8])
    assert e.value.status == b.LS_ERR_NOT_LOADED
    for l in (-1, 0, 1):
        st.load_block(l, blocks[l])
    with pytest.raises(LsError) as e:  # head block still missing
        st.prefill(tok, [8])
    assert e.value.status == b.LS_ERR_NOT_LOADED
    st.load_block(2, blocks[2])
    with pytest.raises(LsError) as e:
        st.load_block(1, blocks[1])
    assert e.value.status == b.LS_ERR_ALREADY_LOADED
    with pytest.raises(LsError) as e:
        st.load_block(3, blocks[1])
    assert e.value.status == b.LS_ERR_BLOCK_RANGE
    with pytest.raises(LsError) as e:  # 17 tokens in one sequence, max_seq 16
        st.prefill(to_dev(shape, synth.token_ids(1, 17, shape.vocab)), [17])
    assert e.value.status == b.LS_ERR_KV_OVERFLOW
    with pytest.raises(LsError) as e:  # 3 sequences, max_batch 2
        st.prefill(tok, [2, 3, 3])
    assert e.value.status == b.LS_ERR_INVALID_ARG
    with pytest.raises(LsError) as e:  # 25 tokens, max_tokens 24
        st.prefill(to_dev(shape, synth.token_ids(1, 25, shape.vocab)), [13, 12])
    assert e.value.status == b.LS_ERR_INVALID_ARG
    with pytest.raises(LsError) as e:
        st.decode(tok[:1], 1, 16)
    assert e.value.status == b.LS_ERR_KV_OVERFLOW
    torch.cuda.synchronize()
    assert (st.seq_lens.cpu() == -7).all()  # no failing call touched the device
    # and the stage still works afterwards; a sequence at max_seq is left alone by decode
    st.prefill(to_dev(shape, synth.token_ids(1, 16, shape.vocab)), [16])
    torch.cuda.synchronize()
    assert st.seq_lens.cpu().tolist() == [16, -7]
    st.reset_blocks()
    with pytest.raises(LsError) as e:
        st.prefill(tok, [8])
    assert e.value.status == b.LS_ERR_NOT_LOADED
    st.close()


def test_layer_times_show_the_gate_and_the_overlap():
    """With profiling on, every layer's kernels end after that layer's block copy ended
    (the gate), copies and layers have positive durations, and completion times rise with
    the layer index."""
    import torch
    from paper_2502_09922_amd import LsError, binding as b

    shape, seed, lengths = MINI_BF16, 13, [100, 60]
    B, S = len(lengths), max(lengths)
    st = make_gpu(shape, seed, 0, 3, B, S + 1, sum(lengths), load=False)
    with pytest.raises(LsError):  # nothing recorded yet
        st.layer_times()
    blocks = {l: st.stage_host_block(l, buf) for l, buf in packed_blocks(st, seed).items()}
    tok = to_dev(shape, synth.token_ids(seed + 1, sum(lengths), shape.vocab))
    st.set_profiling(True)
    copy_stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    for l in st.block_ids():
        st.load_block(l, blocks[l], stream=copy_stream)
    st.prefill(tok, lengths)
    torch.cuda.synchronize()
    lt = st.layer_times()
    assert all(c > 0 for c in lt["copy_ms"]) and all(p > 0 for p in lt["compute_ms"])
    assert all(ce >= cp for ce, cp in zip(lt["compute_end_ms"], lt["copy_end_ms"]))
    assert lt["compute_end_ms"] == sorted(lt["compute_end_ms"])
    assert lt["copy_end_ms"] == sorted(lt["copy_end_ms"])
    # the probe brackets one operator of one layer
    st.probe(b.LS_OP_GEMM_QKV, 1, 0)
    st.prefill(tok, lengths)
    st.prefill(tok, lengths)
    torch.cuda.synchronize()
    times = st.probe_times()
    assert len(times) == 2 and all(t > 0 for t in times)
    st.probe(b.LS_OP_NONE)
    with pytest.raises(LsError):
        st.probe(b.LS_OP_GEMM_QKV, 7, 0)
    st.close()


def test_coarse_blocks_of_several_layers_equal_per_layer_blocks():
    """ls_stage_load_layers: one bulk copy for layers 0..1, another for layer 2, gives the
    same bits as one copy per layer; overlapping or out-of-range requests enqueue nothing."""
    import torch
    from paper_2502_09922_amd import LsError, binding as b

    shape, seed, lengths = MINI_BF16, 9, [40, 7, 90]
    B, S = len(lengths), max(lengths)
    tok = to_dev(shape, synth.token_ids(seed + 1, sum(lengths), shape.vocab))
    pre = make_gpu(shape, seed, 0, 3, B, S + 1, sum(lengths))
    ref_tok, ref_lg = pre.prefill(tok, lengths, want_logits=True)
    st = make_gpu(shape, seed, 0, 3, B, S + 1, sum(lengths), load=False)
    st.slab.view(torch.int16).fill_(0x7FC0)
    packed = packed_blocks(st, seed)
    two = st.stage_host_block(100, np.concatenate([packed[0], packed[1]]))
    copy_stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    with pytest.raises(LsError) as e:
        st.load_layers(1, 3, two, stream=copy_stream)
    assert e.value.status == b.LS_ERR_BLOCK_RANGE
    st.load_block(2, st.stage_host_block(2, packed[2]), stream=copy_stream)
    with pytest.raises(LsError) as e:  # layer 2 is already enqueued: nothing of 1..2 is copied
        st.load_layers(1, 2, two, stream=copy_stream)
    assert e.value.status == b.LS_ERR_ALREADY_LOADED
    st.load_layers(0, 1, two, stream=copy_stream)
    for l in (-1, 3):
        st.load_block(l, st.stage_host_block(l, packed[l]), stream=copy_stream)
    got_tok, got_lg = st.prefill(tok, lengths, want_logits=True)
    torch.cuda.synchronize()
    assert torch.equal(got_lg, ref_lg) and torch.equal(got_tok, ref_tok)
    st.close(); pre.close()


def test_measurement_probes_report_plausible_rates():
    """The roofline aids of bench.py: a streaming read and a register-only MFMA loop.  Their
    values are machine properties; the test only fixes that they run and land above a tenth
    of the published peaks (8 TB/s, 2.5 PFLOP/s) and, for the MFMA loop, not above the peak
    (a 256 MB buffer may be served from the memory-side cache, so the read has no upper bound here)."""
    import ctypes as C
    import torch
    from paper_2502_09922_amd import binding as b

    buf = torch.ones(1 << 28, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    read = b.ls_probe_read_gbps(C.c_void_p(buf.data_ptr()), buf.numel(), 2, C.c_void_p(sink.data_ptr()), st)
    mfma = b.ls_probe_mfma_tflops(500, 2, C.c_void_p(sink.data_ptr()), st)
    assert 800.0 < read < 1e5, read
    assert 250.0 < mfma <= 2500.0 * 1.02, mfma
    assert float(sink.sum()) == 0.0 and int(buf[:64].sum()) == 64  # neither buffer was written
