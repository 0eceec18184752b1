"""Parity at the benchmark's real layer dimensions and in the launch configuration that
bench.py times.

The oracle cannot run a whole 7B stage on 4096 rows in test time, so:
  * at the full bench configuration (8 layers, batch 8 x 512, then decode) the GPU runs
    everything, and the oracle recomputes ONE sequence alone -- causal attention makes a
    sequence's outputs independent of the other sequences in the batch, so every row of
    that sequence (prompt pass and decode steps) is compared element by element;
  * the 13B- and 70B-shaped layers (first / last stage pieces, GQA, LM head at V=32000)
    run as one-layer slices on short ragged batches, compared in full.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

import synth
from helpers import block_tensors, make_gpu, make_oracle, rel_l2, to_dev, to_host
from oracle.stage_oracle import OracleStage

pytestmark = pytest.mark.gpu
TOL = 2e-2


def test_bench_configuration_llama7b_stage_sampled_sequence():
    """Layers 8..15 of the 7B shape, batch 8 x 512 prompt rows, then 3 decode steps: the
    exact launch shapes of the default bench workload.  Sequences 5 and 7 are checked against
    the oracle run on each of them alone (the rows of sequence 7 lie in the last, partial
    round of the gate-up GEMM's tiles); all sequences are checked for finiteness."""
    shape, seed, lo, hi = synth.CONFIGS["llama7b"], 1234, 8, 16
    B, S, steps, picks = 8, 512, 3, (5, 7)
    with ThreadPoolExecutor(8) as ex:
        tensors = dict(zip(range(lo, hi), ex.map(lambda l: synth.layer_tensors(shape, seed, l), range(lo, hi))))
    from paper_2502_09922_amd import Stage, pack_block

    gpu = Stage(shape, lo, hi, B, S + 128, B * S)
    for l in range(lo, hi):
        gpu.load_block(l, gpu.stage_host_block(l, pack_block(gpu.cfg, l, [tensors[l][n] for n in synth.TENSOR_ORDER_LAYER])))
    x = synth.hidden_states(shape, seed + 1, B * S)
    got = to_host(gpu.prefill(to_dev(shape, x), [S] * B))
    assert np.isfinite(got).all()
    dec_in = [synth.hidden_states(shape, seed + 2 + t, B) for t in range(steps)]
    got_dec = [to_host(gpu.decode(to_dev(shape, dec_in[t]), B, S + t)) for t in range(steps)]
    gpu.close()

    for pick in picks:
        ora = OracleStage(shape, lo, hi, 1, S + steps)
        for l in range(lo, hi):
            ora.load_tensors(l, tensors[l])
        want = ora.prefill(x[pick * S : (pick + 1) * S], [S])
        mine = got[pick * S : (pick + 1) * S]
        assert rel_l2(mine, want) <= TOL, pick
        row_err = np.linalg.norm(mine - want, axis=1) / np.linalg.norm(want, axis=1)
        assert row_err.max() <= 2 * TOL, (pick, row_err.argmax(), row_err.max())
        for t in range(steps):
            want_t = ora.decode(dec_in[t][pick : pick + 1])
            assert rel_l2(got_dec[t][pick : pick + 1], want_t) <= TOL, (pick, t)
            assert np.isfinite(got_dec[t]).all()


@pytest.mark.parametrize("name,lo,hi,lengths,steps", [
    ("llama13b", 39, 40, [70, 5, 33], 2),     # last stage piece: layer + final norm + LM head at V=32000
    ("llama13b", 0, 1, [64, 9], 2),           # first stage piece: embedding gather + layer
    ("llama70b", 40, 41, [130, 40, 7, 77], 3),  # grouped-query attention, 64 q heads on 8 kv heads
])
def test_one_layer_slices_at_real_dimensions(name, lo, hi, lengths, steps):
    shape, seed = synth.CONFIGS[name], 77
    B, S, T = len(lengths), max(lengths), sum(lengths)
    gpu = make_gpu(shape, seed, lo, hi, B, S + steps, T)
    ora = make_oracle(shape, seed, lo, hi, B, S + steps)
    if gpu.first:
        x = synth.token_ids(seed + 1, T, shape.vocab)
    else:
        x = synth.hidden_states(shape, seed + 1, T)
    want = ora.prefill(x, lengths)
    if gpu.last:
        tok, lg = gpu.prefill(to_dev(shape, x), lengths, want_logits=True)
        assert rel_l2(to_host(lg), want[1]) <= TOL
        err = np.abs(to_host(lg) - want[1]).max()
        for b in range(B):  # greedy token agrees unless the oracle's top two are a declared tie
            top2 = np.sort(want[1][b])[-2:]
            assert int(tok[b]) == int(want[0][b]) or top2[1] - top2[0] < 4 * err
    else:
        assert rel_l2(to_host(gpu.prefill(to_dev(shape, x), lengths)), want) <= TOL
    for t in range(steps):
        if gpu.first:
            xs = synth.token_ids(seed + 2 + t, B, shape.vocab)
        else:
            xs = synth.hidden_states(shape, seed + 2 + t, B)
        want = ora.decode(xs)
        if gpu.last:
            _, lg = gpu.decode(to_dev(shape, xs), B, S + t, want_logits=True)
            assert rel_l2(to_host(lg), want[1]) <= TOL
        else:
            assert rel_l2(to_host(gpu.decode(to_dev(shape, xs), B, S + t)), want) <= TOL
    gpu.close()


@pytest.mark.parametrize("batch", [13, 16, 17, 20, 40, 64])
def test_decode_with_many_sequences(batch):
    """Decode batches of 17..64 rows take the wider weight-streaming kernel variants; 13 and
    16 rows are the upper end of the narrow one (every wavefront owns rows of the folded norm)."""
    shape, seed, steps = synth.StageShape("bf16", 2, 512, 8, 2, 64, 1408, 0), 31, 3
    lengths = [int(n) for n in synth.ragged_lengths(seed, batch, 1, 12)]
    S, T = max(lengths), sum(lengths)
    gpu = make_gpu(shape, seed, 0, 2, batch, S + steps, T)
    ora = make_oracle(shape, seed, 0, 2, batch, S + steps)
    x = synth.hidden_states(shape, seed + 1, T)
    assert rel_l2(to_host(gpu.prefill(to_dev(shape, x), lengths)), ora.prefill(x, lengths)) <= TOL
    for t in range(steps):
        xs = synth.hidden_states(shape, seed + 2 + t, batch)
        got, want = to_host(gpu.decode(to_dev(shape, xs), batch, S + t)), ora.decode(xs)
        assert rel_l2(got, want) <= TOL
        row_err = np.linalg.norm(got - want, axis=1) / np.linalg.norm(want, axis=1)
        assert row_err.max() <= 3 * TOL
    gpu.close()


@pytest.mark.parametrize("name,layer,batch,prompt,picks", [
    # bench slices of the larger configurations, one layer of each at the full batch: the
    # launch shapes bench.py times (many-row prompt GEMMs, decode with 32 / 64 rows, ragged
    # contexts up to 2048 keys for the grouped-query decode attention)
    ("llama13b", 16, 32, 1024, (0, 21)),
    ("llama70b", 40, 64, (128, 2048), (3, "longest")),
])
def test_bench_slices_of_the_larger_configurations_sampled_sequences(name, layer, batch, prompt, picks):
    """The GPU runs the whole batch; the oracle recomputes the picked sequences alone
    (a sequence's rows do not depend on the other sequences of the batch) for the prompt
    pass and two decode steps."""
    import bench

    shape, seed, steps = synth.CONFIGS[name].with_(vocab=0), 1234, 2
    lengths = bench.prompt_lengths(synth, batch, prompt)
    B, S, T = len(lengths), max(lengths), sum(lengths)
    tensors = synth.layer_tensors(shape, seed, layer)
    from paper_2502_09922_amd import Stage, pack_block

    gpu = Stage(shape, layer, layer + 1, B, S + steps, T)
    gpu.load_block(layer, gpu.stage_host_block(layer, pack_block(gpu.cfg, layer, [tensors[n] for n in synth.TENSOR_ORDER_LAYER])))
    x = synth.hidden_states(shape, seed + 1, T)
    got = to_host(gpu.prefill(to_dev(shape, x), lengths))
    assert np.isfinite(got).all()
    dec_in = [synth.hidden_states(shape, seed + 2 + t, B) for t in range(steps)]
    got_dec = [to_host(gpu.decode(to_dev(shape, dec_in[t]), B, S + t)) for t in range(steps)]
    assert gpu.seq_lens.cpu().numpy()[:B].tolist() == [n + steps for n in lengths]
    gpu.close()
    off = np.concatenate([[0], np.cumsum(lengths)])
    for pick in picks:
        b = int(np.argmax(lengths)) if pick == "longest" else pick
        ora = OracleStage(shape, layer, layer + 1, 1, lengths[b] + steps)
        ora.load_tensors(layer, tensors)
        want = ora.prefill(x[off[b]:off[b + 1]], [lengths[b]])
        mine = got[off[b]:off[b + 1]]
        assert rel_l2(mine, want) <= TOL, (b, rel_l2(mine, want))
        row_err = np.linalg.norm(mine - want, axis=1) / np.linalg.norm(want, axis=1)
        assert row_err.max() <= 2 * TOL, (b, row_err.argmax(), row_err.max())
        for t in range(steps):
            want_t = ora.decode(dec_in[t][b:b + 1])
            assert rel_l2(got_dec[t][b:b + 1], want_t) <= TOL, (b, t)
            assert np.isfinite(got_dec[t]).all()
