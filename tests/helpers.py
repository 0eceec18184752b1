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
# ... and their element-level companions.  u is the resolution of the stored output: 2^-8 for
# bf16 (one rounding of a value v is at most 2^-9 |v|), 2^-20 for the fp32 path (fp32 accumulation
# against fp64).  Two bounds per element:
#   tail:   |got - want| <= u |want| + TAIL * rms(row of got - want): beyond the rounding of the
#           stored value itself, no element may stick out of its own row's error level.  Errors
#           of the bf16 hand-offs between kernels add up like a Gaussian, whose largest of
#           10^6..10^8 samples sits near 5.5 standard deviations; rows whose error level varies
#           across columns by 1.5x reach 8.  An isolated wrong element is caught from about a
#           tenth of the output's scale downwards, however little it moves the L2 norms.
#   scale:  |got - want| <= K_ELEM u rms(want): a Gaussian error at the stated tolerance itself
#           (2e-2) peaks at 5.7 x 2e-2 x 256 u = 29 u; the largest measured anywhere is 17 u (the
#           8-layer 7B stage).  A wholly wrong element is off by about rms(want) = 256 u.
U_ELEM = {"f32": 2.0**-20, "bf16": 2.0**-8}
TAIL = 10.0
K_ELEM = 40.0
ROW_FACTOR = 2.0   # no single row's relative L2 error above ROW_FACTOR * TOL
COL_FACTOR = 2.0   # no single column's error (over >= 16 rows, against rms(want)) above COL_FACTOR * TOL


def check_close(got, want, dtype, what="", tail=None):
    """Compare one output [rows, cols] with the oracle's: relative L2 over the whole output
    (the stated tolerance), per row, per column, and element by element.  Prints what it
    measured, then asserts.  `tail` overrides TAIL for outputs whose element errors are not
    sums of many terms (see the callers)."""
    got = np.asarray(got, np.float64).reshape(np.shape(want))
    want = np.asarray(want, np.float64)
    if want.ndim == 1:
        got, want = got[None, :], want[None, :]
    diff = got - want
    u = U_ELEM[dtype]
    rms = float(np.sqrt(np.mean(want * want)))
    row_rms = np.sqrt(np.mean(diff * diff, axis=1, keepdims=True))
    excess = np.maximum(np.abs(diff) - u * np.abs(want), 0.0) / np.maximum(row_rms, u * rms / 16)
    m = {
        "rel_l2": float(np.linalg.norm(diff) / np.linalg.norm(want)),
        "row": float((np.linalg.norm(diff, axis=1) / np.linalg.norm(want, axis=1)).max()),
        "col": float((np.linalg.norm(diff, axis=0) / (rms * math.sqrt(want.shape[0]))).max()),
        "elem": float(np.abs(diff).max() / rms),
        "tail": float(excess.max()),
    }
    print("parity %-56s rows %5d  rel-L2 %.2e  worst row %.2e  column %.2e  element %.2e rms (%.1f u), %.1f sigma of its row"
          % (str(what)[:56], want.shape[0], m["rel_l2"], m["row"], m["col"], m["elem"], m["elem"] / u, m["tail"]))
    assert np.isfinite(got).all(), what
    assert m["rel_l2"] <= TOL[dtype], (what, m)
    assert m["row"] <= ROW_FACTOR * TOL[dtype], (what, m, int((np.linalg.norm(diff, axis=1) / np.linalg.norm(want, axis=1)).argmax()))
    if want.shape[0] >= 16:
        assert m["col"] <= COL_FACTOR * TOL[dtype], (what, m, int(np.linalg.norm(diff, axis=0).argmax()))
    assert m["tail"] <= (TAIL if tail is None else tail), (what, m, np.unravel_index(excess.argmax(), diff.shape))
    assert m["elem"] <= K_ELEM * u, (what, m, np.unravel_index(np.abs(diff).argmax(), diff.shape))
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
