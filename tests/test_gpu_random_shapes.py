"""Parity over a seeded sweep of small bf16 stage shapes: hidden sizes, head layouts (one to
eight query heads per kv head, head_dim 64 and 128), FFN widths, batch sizes on both sides of
every kernel-choice boundary (1..64 rows) and ragged prompts from one token up.  Every case
runs a prompt pass and three decode steps through the C ABI and is compared with the oracle
(relative L2 over the output, per row, per column, and the largest element error)."""
import numpy as np
import pytest

import synth
from helpers import check_close, check_delta, make_gpu, make_oracle, to_dev, to_host
from oracle.stage_oracle import decode_values

pytestmark = pytest.mark.gpu


def cases(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        hd = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 3, 4, 8])) if hd == 128 else int(rng.choice([1, 2, 4]))
        d = int(rng.choice([256, 384, 512, 640, 768, 1024, 1536]))
        ffn = int(rng.choice([256, 688, 1024, 1408, 2048]))
        layers = int(rng.choice([1, 2]))
        batch = int(rng.choice([1, 2, 3, 5, 8, 9, 13, 16, 17, 24, 33, 48, 64]))
        lengths = [int(x) for x in rng.integers(1, 70, size=batch)]
        yield synth.StageShape("bf16", layers, d, hkv * group, hkv, hd, ffn, 0), lengths, int(rng.integers(0, 10000))


@pytest.mark.parametrize("sweep_seed", [1, 2])
def test_seeded_sweep_of_shapes_batches_and_ragged_lengths(sweep_seed):
    steps = 3
    for shape, lengths, seed in cases(sweep_seed, 30):
        B, S, T = len(lengths), max(lengths), sum(lengths)
        what = (shape, B, T, seed)
        gpu = make_gpu(shape, seed, 0, shape.n_layers_total, B, S + steps, T)
        ora = make_oracle(shape, seed, 0, shape.n_layers_total, B, S + steps)
        x = synth.hidden_states(shape, seed + 1, T)
        tag = "d%d F%d Hq%d/Hkv%d hd%d L%d B%d T%d" % (shape.hidden, shape.ffn, shape.n_q_heads, shape.n_kv_heads,
                                                        shape.head_dim, shape.n_layers_total, B, T)
        got, want = to_host(gpu.prefill(to_dev(shape, x), lengths)), ora.prefill(x, lengths)
        check_close(got, want, "bf16", tag + " prompt")
        check_delta(got, want, decode_values(x), "bf16", tag + " prompt")
        for t in range(steps):
            xs = synth.hidden_states(shape, seed + 2 + t, B)
            got, want = to_host(gpu.decode(to_dev(shape, xs), B, S + t)), ora.decode(xs)
            check_close(got, want, "bf16", tag + " step %d" % t)
        gpu.close()


def whole_model_cases(seed, n):
    rng = np.random.default_rng(seed)
    for _ in range(n):
        dtype = str(rng.choice(["bf16", "bf16", "f32"]))
        hd = int(rng.choice([64, 128]))
        hkv = int(rng.choice([1, 2]))
        group = int(rng.choice([1, 2, 4]))
        d = int(rng.choice([256, 512, 768]))
        ffn = int(rng.choice([256, 688, 1408]))
        vocab = int(rng.choice([512, 1000, 4096]))
        batch = int(rng.choice([1, 3, 8, 17, 20]))
        lengths = [int(x) for x in rng.integers(1, 40, size=batch)]
        yield synth.StageShape(dtype, 2, d, hkv * group, hkv, hd, ffn, vocab), lengths, int(rng.integers(0, 10000))


def test_seeded_sweep_of_whole_models_with_embedding_and_head():
    """Embedding gather, layers, final norm, LM head and greedy argmax as one stage, fp32 and
    bf16: logits against the oracle, greedy tokens teacher-forced and tie-adjusted."""
    from helpers import TOL as TOLS
    from test_gpu_parity import run_full_model

    for shape, lengths, seed in whole_model_cases(5, 16):
        errs, agree = run_full_model(shape, seed, lengths, 2)
        assert max(errs) <= TOLS[shape.dtype], (shape, lengths, seed, errs)
        adj = sum(a[1] for a in agree)
        n = sum(a[2] for a in agree)
        assert adj >= 0.99 * n, (shape, lengths, seed, agree)
