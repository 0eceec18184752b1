"""Shared test plumbing: the same seeded tensors go to the HIP stage and to the oracle."""
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


def greedy_agreement(tok_gpu, logits_gpu, tok_ora, logits_ora):
    """(raw matches, tie-adjusted matches, count)."""
    err = np.abs(logits_gpu - logits_ora).max()
    raw = adj = 0
    for b in range(len(tok_ora)):
        top2 = np.sort(logits_ora[b])[-2:]
        tie = (top2[1] - top2[0]) < 4 * err
        ok = int(tok_gpu[b]) == int(tok_ora[b])
        raw += ok
        adj += ok or tie
    return raw, adj, len(tok_ora)
