"""Mode switching by KV-cache recomputation (Section 4.4): a node that has received the whole
model leaves the execution pipeline and serves its requests locally; its cache for all layers
is rebuilt by one prompt pass over prompt + tokens generated so far, instead of moving the
stages' caches.  Checked here: the rebuilt cache equals the caches the pipeline's stages built
token by token (same values up to bf16 rounding: the prompt-pass and the decode kernels round
in different places), the recomputing pass predicts the token the pipeline produced next, and
generation continues in local mode with logits that match both the pipeline's continuation
and the CPU oracle."""
import numpy as np
import pytest

import synth
from helpers import check_close, greedy_agreement, make_gpu, make_oracle, rel_l2, to_dev, to_host

pytestmark = pytest.mark.gpu

SHAPE = synth.StageShape("bf16", 4, 512, 8, 2, 64, 1408, 1000)
SEED = 41


def cache_rows(shape, k_bytes, n_layers, max_b, max_s, b, n):
    """[layers][kv heads][n][hd] float64 view of sequence b's first n cached positions."""
    import torch

    t = k_bytes.view(torch.bfloat16).view(n_layers, max_b, shape.n_kv_heads, max_s, shape.head_dim)
    return t[:, b, :, :n, :].double().cpu().numpy()


def test_recomputed_cache_equals_the_pipeline_built_cache_and_generation_continues():
    import torch
    from paper_2502_09922_amd import MicroBatch, Pipeline

    lengths, gen, more = [40, 7, 90, 23], 5, 3
    B, S = len(lengths), max(lengths)
    max_s, max_t = S + gen + more + 1, sum(lengths) + B * gen
    L, cut = SHAPE.n_layers_total, 2
    a = make_gpu(SHAPE, SEED, 0, cut, B, max_s, max_t)
    b = make_gpu(SHAPE, SEED, cut, L, B, max_s, max_t)
    pipe = Pipeline([a, b])
    mb = MicroBatch(pipe, max_t)
    prompt = synth.token_ids(SEED + 1, sum(lengths), SHAPE.vocab)

    # pipelined mode: prompt pass + `gen` generation steps; tokens[t][b] is the t-th new token
    tokens = [pipe.run(0, [mb], [to_dev(SHAPE, prompt)], lengths=[lengths])[0]]
    for t in range(gen):
        tokens.append(pipe.run(1, [mb], [tokens[-1]], max_ctx=[S + t])[0])
    torch.cuda.synchronize()
    tok_h = [t.cpu().numpy() for t in tokens]

    # mode switch: the whole model as one local stage; each request's available tokens are its
    # prompt and the first `gen` generated tokens (the last one, tokens[gen], is the next input)
    whole = make_gpu(SHAPE, SEED, 0, L, B, max_s, max_t)
    off = np.concatenate([[0], np.cumsum(lengths)])
    seqs = [np.concatenate([prompt[off[i]:off[i + 1]], [tok_h[t][i] for t in range(gen)]]).astype(np.int32)
            for i in range(B)]
    new_len = [len(s) for s in seqs]
    nxt, lg_re = whole.prefill(to_dev(SHAPE, np.concatenate(seqs)), new_len, want_logits=True)
    torch.cuda.synchronize()
    assert whole.seq_lens.cpu().tolist() == new_len

    # (1) the rebuilt cache holds what the stages built step by step
    for i in range(B):
        n = new_len[i]
        for name, wt, parts in (("k", whole.k, (mb.caches[0][0], mb.caches[1][0])),
                                ("v", whole.v, (mb.caches[0][1], mb.caches[1][1]))):
            got = cache_rows(SHAPE, wt, L, B, max_s, i, n)
            want = np.concatenate([cache_rows(SHAPE, parts[0], cut, B, max_s, i, n),
                                   cache_rows(SHAPE, parts[1], L - cut, B, max_s, i, n)])
            assert rel_l2(got, want) <= 1e-2, (name, i, rel_l2(got, want))

    # (2) the recomputing pass predicts the token the pipeline produced for that position, and
    # both agree with the oracle run over the same token sequence
    ora = make_oracle(SHAPE, SEED, 0, L, B, max_s)
    nt_o, lg_o = ora.prefill(np.concatenate(seqs), new_len)
    check_close(to_host(lg_re), lg_o, "bf16", "logits after the cache was recomputed")
    _, adj, n = greedy_agreement(nxt.cpu().numpy(), to_host(lg_re), nt_o, lg_o)
    assert adj == n
    _, adj, n = greedy_agreement(tok_h[gen], to_host(lg_re), nt_o, lg_o)
    assert adj == n

    # (3) generation continues locally; the pipeline continues too: same logits within tolerance
    feed = tokens[gen]
    for t in range(more):
        (p_tok,), (p_lg,) = pipe.run(1, [mb], [feed], max_ctx=[S + gen + t], want_logits=True)
        w_tok, w_lg = whole.decode(feed, B, S + gen + t, want_logits=True)
        nt_o, lg_o = ora.decode(feed.cpu().numpy().astype(np.int32))
        torch.cuda.synchronize()
        assert rel_l2(to_host(w_lg), to_host(p_lg)) <= 2e-2
        check_close(to_host(w_lg), lg_o, "bf16", "continued generation")
        _, adj, n = greedy_agreement(w_tok.cpu().numpy(), to_host(w_lg), nt_o, lg_o)
        assert adj == n
        feed = to_dev(SHAPE, nt_o.astype(np.int32))  # teacher forcing for all three
    pipe.close()
    for st in (a, b, whole):
        st.close()
