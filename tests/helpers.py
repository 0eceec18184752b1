"""Shared test plumbing: the same seeded tensors go to the HIP stage and to the oracle."""
import math

import numpy as np

import synth
from oracle.stage_oracle import OracleStage, decode_values


def block_tensors(shape, seed, layer):
    """(tensors dict, order) of block `layer` from the seeded generator."""
    if layer == -1:
        return synth.embed_tensors(shape, seed), ("embed",)
    if layer == shape.n_layers_total:
        return synth.head_tensors(shape, seed), synth.TENSOR_ORDER_HEAD
    return synth.layer_tensors(shape, seed, layer), synth.TENSOR_ORDER_LAYER


def make_oracle(shape, seed, lo, hi, max_batch, max_seq):
    st = OracleStage(shape, lo, hi, max_batch, max_seq)
    ids = ([-1] if st.first else []) + list(range(lo, hi)) + ([shape.n_layers_total] if st.last else [])
    for layer in ids:
        st.load_tensors(layer, block_tensors(shape, seed, layer)[0])
    return st


def packed_blocks(stage, seed):
    """layer -> packed uint8 numpy block, through the product's own format function."""
    from paper_2502_09922_amd import pack_block

    out = {}
    for layer in stage.block_ids():
        t, order = block_tensors(stage.shape, seed, layer)
        out[layer] = pack_block(stage.cfg, layer, [t[n] for n in order])
    return out


def make_gpu(shape, seed, lo, hi, max_batch, max_seq, max_tokens, load=True):
    from paper_2502_09922_amd import Stage

    st = Stage(shape, lo, hi, max_batch, max_seq, max_tokens)
    if load:
        for layer, buf in packed_blocks(st, seed).items():
            st.load_block(layer, st.stage_host_block(layer, buf))
    return st


def to_dev(shape, a):
    """numpy storage-format array (fp32, bf16 bits as uint16, int32 ids) -> device tensor."""
    import torch

    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    """device tensor -> float64 numpy."""
    return t.detach().to("cpu").double().numpy()


def rel_l2(got, want):
    return float(np.linalg.norm(np.asarray(got, np.float64) - want) / np.linalg.norm(want))


# Tolerances of the benchmark definition (relative L2 over an output) ...
TOL = {"f32": 1e-4, "bf16": 2e-2}
# ... and their element-level companions.  An output element's error is bounded against the
# output's own scale: |got - want| <= K_ELEM * u * rms(want), u = 2^-8 for bf16 storage (one
# rounding of a value near rms is at most 2^-9 rms; errors of the bf16 hand-offs between kernels
# add up over the layers roughly like a Gaussian of standard deviation rel_l2 * rms, whose largest
# of 10^6..10^8 samples sits near 5.5 standard deviations) and 2^-20 for the fp32 path (fp32
# accumulation against fp64).  A wholly wrong element is off by about rms, i.e. 256 u.
U_ELEM = {"f32": 2.0**-20, "bf16": 2.0**-8}
K_ELEM = 12.0
ROW_FACTOR = 2.0   # no single row's relative L2 error above ROW_FACTOR * TOL
COL_FACTOR = 2.0   # no single column's error (over >= 16 rows, against rms(want)) above COL_FACTOR * TOL


def check_close(got, want, dtype, what=""):
    """Compare one output [rows, cols] with the oracle's: relative L2 over the whole output
    (the stated tolerance), per row, per column, and the largest element error against the
    output's scale.  Prints what it measured, then asserts."""
    got = np.asarray(got, np.float64).reshape(np.shape(want))
    want = np.asarray(want, np.float64)
    if want.ndim == 1:
        got, want = got[None, :], want[None, :]
    diff = got - want
    rms = float(np.sqrt(np.mean(want * want)))
    m = {
        "rel_l2": float(np.linalg.norm(diff) / np.linalg.norm(want)),
        "row": float((np.linalg.norm(diff, axis=1) / np.linalg.norm(want, axis=1)).max()),
        "col": float((np.linalg.norm(diff, axis=0) / (rms * math.sqrt(want.shape[0]))).max()),
        "elem": float(np.abs(diff).max() / rms),
    }
    print("parity %-58s rows %5d  rel-L2 %.2e  worst row %.2e  worst column %.2e  max|err|/rms %.2e (%.1f u)"
          % (str(what)[:58], want.shape[0], m["rel_l2"], m["row"], m["col"], m["elem"], m["elem"] / U_ELEM[dtype]))
    assert np.isfinite(got).all(), what
    assert m["rel_l2"] <= TOL[dtype], (what, m)
    assert m["row"] <= ROW_FACTOR * TOL[dtype], (what, m, int((np.linalg.norm(diff, axis=1) / np.linalg.norm(want, axis=1)).argmax()))
    if want.shape[0] >= 16:
        assert m["col"] <= COL_FACTOR * TOL[dtype], (what, m, int(np.linalg.norm(diff, axis=0).argmax()))
    assert m["elem"] <= K_ELEM * U_ELEM[dtype], (what, m, np.unravel_index(np.abs(diff).argmax(), diff.shape))
    return m


def check_delta(got_out, want_out, x_in, dtype, what=""):
    """The stage's own contribution, out - in, row by row: in `out` the input residual dominates
    each row's norm, so a partly wrong attention or FFN term shows far more clearly here.  The
    bound is the stated tolerance relative to the delta's scale plus the rounding of `out`
    itself (its bf16 storage rounds the whole row, input part included)."""
    got_d = np.asarray(got_out, np.float64) - x_in
    want_d = np.asarray(want_out, np.float64) - x_in
    err = np.linalg.norm(got_d - want_d, axis=1)
    floor = U_ELEM[dtype] / 2 * np.linalg.norm(want_out, axis=1)  # rounding of the stored output row
    rel = (np.maximum(err - floor, 0.0) / np.linalg.norm(want_d, axis=1)).max()
    print("parity %-58s delta rows: worst relative error %.2e (|delta|/|out| %.2f)"
          % (str(what)[:58], rel, float(np.linalg.norm(want_d) / np.linalg.norm(want_out))))
    assert rel <= ROW_FACTOR * TOL[dtype], (what, rel)
    return rel


def greedy_agreement(tok_gpu, logits_gpu, tok_ora, logits_ora, dtype="bf16"):
    """(raw matches, tie-adjusted matches, count).  A mismatch counts as a declared tie only if
    the token the GPU chose is one the oracle itself ranks within 4 x that row's own logit
    error of its top-1 (the error is capped at 4 x TOL x the row's rms, so a badly wrong row
    cannot widen its own window)."""
    raw = adj = 0
    for b in range(len(tok_ora)):
        lo = np.asarray(logits_ora[b], np.float64)
        err = min(float(np.abs(np.asarray(logits_gpu[b], np.float64) - lo).max()),
                  4 * TOL[dtype] * float(np.sqrt(np.mean(lo * lo))))
        g, o = int(tok_gpu[b]), int(tok_ora[b])
        ok = g == o
        tie = (not ok) and 0 <= g < lo.size and lo[o] - lo[g] <= 4 * err
        raw += ok
        adj += ok or tie
    return raw, adj, len(tok_ora)
