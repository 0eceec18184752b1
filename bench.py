"""Benchmark of the stage hot path on one MI355X.

One step = one pass of the whole hot path over one batch: the prompt pass of the stage
followed by the KV-cached decode steps of the workload, weights resident in HBM.

Default workload: the Llama-13B-shaped FULL model as one stage (benchmark configuration 3, the
largest configuration that is a whole model on one GPU): embedding, 40 layers, final norm and
LM head at V = 32000, batch 32 x 1024 prompt token ids, then 64 greedy decode steps, each fed
with the tokens the step before produced.  The other configurations ride along as extra
keys of the same JSON line (`other_workloads`): the 7B-shaped middle stage (configuration 2),
the 70B-shaped grouped-query stage on 64 ragged prompts and 256 steps (configuration 4) and
execute-while-load of the 7B-shaped full model (configuration 5, `execute_while_load`).

Weights and inputs are seeded synthetic data of the benchmark's recipe (matrices N(0, 0.02),
gains 1 + N(0, 0.02), token ids uniform, hidden states N(0, 1), ragged lengths uniform on
[128, 2048]).  For these throughput runs they are drawn on the device with torch's generator
straight into the weight slab (26-34 GB would take minutes to draw on the host) and adopted
by the stage as blocks that are already in GPU memory; the parity tests draw theirs on the
host (synth/) and send them through the loader.

Prints ONE JSON line.  `value` is tokens handled per second over the whole step (prompt tokens
+ generated tokens, divided by the step time).
"""
import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TF = 2500.0  # MI355X published dense bf16 MFMA rate

WORKLOADS = {
    # name: (shape key, layer_lo, layer_hi, batch, prompt, decode steps)
    "llama13b_full_l0_40_b32_s1024_d64": ("llama13b", 0, 40, 32, 1024, 64),
    "llama70b_stage_l20_40_b64_ragged128_2048_d256": ("llama70b", 20, 40, 64, (128, 2048), 256),
    "llama7b_stage_l8_16_b8_s512_d128": ("llama7b", 8, 16, 8, 512, 128),
    "tiny_f32_b1_s32_d8": ("tiny_f32", 0, 2, 1, 32, 8),
    # slices of the larger configurations (fewer layers, same per-layer shapes)
    "llama13b_l4_b32_s1024_d16": ("llama13b", 16, 20, 32, 1024, 16),
    "llama70b_l4_b64_ragged128_2048_d16": ("llama70b", 40, 44, 64, (128, 2048), 16),
    # execute-while-load: the whole 7B-shaped model streams in as 34 blocks while prefill runs
    "ewl_llama7b_full_b16_s512_d32": ("llama7b", 0, 32, 16, 512, 32),
    # same model, a prompt batch heavy enough that compute, not the host link, is the longer leg
    "ewl_llama7b_full_b64_s512_d32": ("llama7b", 0, 32, 64, 512, 32),
}
DEFAULT = "llama13b_full_l0_40_b32_s1024_d64"
EXTRAS = ("llama7b_stage_l8_16_b8_s512_d128", "llama70b_stage_l20_40_b64_ragged128_2048_d256")
EWL = "ewl_llama7b_full_b16_s512_d32"
SEED = 1234
IDLE_BEFORE_EXTRA_S = 10.0


def prompt_lengths(synth, batch, prompt):
    """Uniform prompts, or (lo, hi): seeded ragged lengths uniform on [lo, hi]."""
    if isinstance(prompt, tuple):
        return [int(n) for n in synth.ragged_lengths(SEED + 7, batch, prompt[0], prompt[1])]
    return [prompt] * batch


def st_block_bytes(st, layer):
    from paper_2502_09922_amd import binding as b

    return b.ls_stage_block_bytes(st.handle, layer)


def build_stage(synth, Stage, pack_block, shape, lo, hi, lengths, steps):
    """Stage + its packed blocks in pinned host memory, drawn on the host (synth/)."""
    import torch

    st = Stage(shape, lo, hi, len(lengths), max(lengths) + steps, sum(lengths))

    def make(layer):
        if layer == -1:
            t, order = synth.embed_tensors(shape, SEED), ("embed",)
        elif layer == shape.n_layers_total:
            t, order = synth.head_tensors(shape, SEED), synth.TENSOR_ORDER_HEAD
        else:
            t, order = synth.layer_tensors(shape, SEED, layer), synth.TENSOR_ORDER_LAYER
        host = torch.empty(int(st_block_bytes(st, layer)), dtype=torch.uint8, pin_memory=True)
        pack_block(st.cfg, layer, [t[n] for n in order], out=host.numpy())
        return layer, host

    with ThreadPoolExecutor(max_workers=8) as ex:
        blocks = dict(ex.map(make, st.block_ids()))
    return st, blocks


def fill_blocks_on_device(st, seed):
    """Draw every block of the stage on the device, in place in the slab, and adopt it: matrices
    and embeddings N(0, 0.02), gains 1 + N(0, 0.02), in the stage's storage type."""
    import ctypes as C

    import torch
    from paper_2502_09922_amd import binding as B

    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    L = st.shape.n_layers_total
    off, nb = C.c_size_t(), C.c_size_t()
    for layer in st.block_ids():
        view = st.block_view(layer)
        for i in range(B.ls_block_tensor_count(C.byref(st.cfg), layer)):
            B.check(B.ls_block_tensor(C.byref(st.cfg), layer, i, C.byref(off), C.byref(nb)))
            t = view[off.value : off.value + nb.value].view(st.tdtype)
            gain = (0 <= layer < L and i in (0, 3)) or (layer == L and i == 0)
            t.normal_(mean=1.0 if gain else 0.0, std=0.02, generator=g)
        st.adopt_block(layer)
    torch.cuda.synchronize()


def device_inputs(torch, st, shape, lengths, dsteps, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    T, B = sum(lengths), len(lengths)
    if st.first:
        x = torch.randint(0, shape.vocab, (T,), dtype=torch.int32, device="cuda", generator=g)
        xd = [torch.randint(0, shape.vocab, (B,), dtype=torch.int32, device="cuda", generator=g) for _ in range(dsteps)]
    else:
        x = torch.empty(T, shape.hidden, dtype=st.tdtype, device="cuda").normal_(generator=g)
        xd = [torch.empty(B, shape.hidden, dtype=st.tdtype, device="cuda").normal_(generator=g) for _ in range(dsteps)]
    return x, xd


def algorithmic_work(st, shape, lo, hi, lengths, dsteps):
    """Flops of the prompt pass and bytes of the decode steps that the method itself needs."""
    T, B, L = sum(lengths), len(lengths), hi - lo
    d, F, e = shape.hidden, shape.ffn, shape.itemsize
    p_mm = shape.qkv_rows * d + d * shape.n_q_heads * shape.head_dim + 3 * F * d
    pre_flops = 2.0 * T * p_mm * L + sum(2.0 * shape.n_q_heads * shape.head_dim * n * (n + 1) for n in lengths) * L
    wbytes = sum(st_block_bytes(st, l) for l in range(lo, hi))
    if st.last:
        pre_flops += 2.0 * B * shape.vocab * d
        wbytes += st_block_bytes(st, shape.n_layers_total)  # final gain + LM head, read once per step
    kv_tok = 2 * shape.n_kv_heads * shape.head_dim * e
    dec_bytes = sum(wbytes + (T + B * (t + 1)) * kv_tok * L for t in range(dsteps))
    return pre_flops, dec_bytes


def stats(v):
    v = sorted(v)
    return {"mean": float(np.mean(v)), "median": float(np.median(v)), "min": float(v[0])}


def run_throughput(name, steps, warmup, probes=True, peaks=False, decode_steps=None):
    """Time `steps` steps of workload `name` (after `warmup`), weights resident.  Returns the
    per-phase numbers and, if asked, the live per-kernel probes."""
    import torch

    import synth
    from paper_2502_09922_amd import Stage, binding as B

    key, lo, hi, batch, prompt, dsteps = WORKLOADS[name]
    if decode_steps is not None:
        dsteps = decode_steps
    shape = synth.CONFIGS[key]
    if not (lo == 0 and hi == shape.n_layers_total):
        shape = shape.with_(vocab=0) if not (lo == 0 or hi == shape.n_layers_total) else shape
    lengths = prompt_lengths(synth, batch, prompt)
    T, max_len = sum(lengths), max(lengths)
    t_gen = time.perf_counter()
    st = Stage(shape, lo, hi, batch, max_len + dsteps, T)
    fill_blocks_on_device(st, SEED)
    x_prefill, x_decode = device_inputs(torch, st, shape, lengths, dsteps, SEED + 1)
    t_gen = time.perf_counter() - t_gen
    stream = torch.cuda.current_stream()
    out = {"workload": name, "layers": [lo, hi], "batch": batch,
           "prompt": prompt if isinstance(prompt, int) else {"ragged": list(prompt), "total_tokens": T, "longest": max_len},
           "decode_steps": dsteps, "steps": steps, "warmup": warmup, "setup_s": round(t_gen, 1),
           "feeds_back_tokens": bool(st.first and st.last)}

    if peaks:
        import ctypes
        cur = ctypes.c_void_p(stream.cuda_stream)
        sink = torch.zeros(4, dtype=torch.float32, device="cuda")
        n = min(st.slab.numel(), 4 << 30)
        peak_read = B.ls_probe_read_gbps(ctypes.c_void_p(st.slab.data_ptr()), n, 3, ctypes.c_void_p(sink.data_ptr()), cur)
        # 50000 iterations are about 7 ms: the rate the chip sustains under its power limit, not a burst
        peak_mfma = B.ls_probe_mfma_tflops(50000, 3, ctypes.c_void_p(sink.data_ptr()), cur)
        assert peak_read > 0 and peak_mfma > 0, B.ls_last_error()
        out["measured_peaks"] = {"read_gbytes_per_s": peak_read, "mfma_bf16_tflops": peak_mfma,
                                 "how": "ls_probe_read_gbps over 4 GiB of the resident weight slab, ls_probe_mfma_tflops (register-only loop of the prompt GEMM's MFMA instruction, varied operands, about 7 ms per repetition)"}

    chain = st.first and st.last  # a whole model: every decode step consumes the previous step's tokens
    out_dec = [(torch.empty(batch, dtype=torch.int32, device="cuda") if st.last
                else torch.empty(batch, shape.hidden, dtype=st.tdtype, device="cuda")) for _ in range(2)]
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    mid_layer = (lo + hi) // 2
    PROBED = min(16, dsteps)  # decode steps per step whose gate-up launch is probed
    probes = probes and dsteps > 0
    probe_lo = (dsteps - PROBED) // 2
    probe_hi = probe_lo + PROBED

    def one_step(timed):
        if timed:
            ev[0].record(stream)
        first = st.prefill(x_prefill, lengths)
        if timed:
            ev[1].record(stream)
        feed = first if chain else None
        for t in range(dsteps):
            # the probe (runtime-stamped start/stop events on one layer's gate-up launch) costs
            # a few microseconds per probed launch: it is on for PROBED decode steps of a step
            if timed and probes and t == probe_lo:
                st.probe(B.LS_OP_GEMM_GATEUP, mid_layer, 1)
            if timed and probes and t == probe_hi:
                st.probe(B.LS_OP_NONE)
            feed = st.decode(feed if chain else x_decode[t], batch, max_len + t, out=out_dec[t & 1])
        if timed:
            ev[2].record(stream)

    for _ in range(warmup):
        one_step(False)
    torch.cuda.synchronize()

    t_pre, t_dec, t_wall, probe_dec, dec_exact = [], [], [], [], True
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ts = time.perf_counter()
        one_step(True)
        torch.cuda.synchronize()
        t_wall.append((time.perf_counter() - ts) * 1e3)
        t_pre.append(ev[0].elapsed_time(ev[1]))
        t_dec.append(ev[1].elapsed_time(ev[2]))
        if probes:
            probe_dec.extend(st.probe_times())
            dec_exact = dec_exact and st.probe_is_kernel_exact()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    st.probe(B.LS_OP_NONE)

    pre_flops, dec_bytes = algorithmic_work(st, shape, lo, hi, lengths, dsteps)
    ms_step = wall * 1e3 / steps
    pre, dec = stats(t_pre), stats(t_dec)
    tokens = T + batch * dsteps
    out.update({
        "tokens_per_step": tokens, "ms_per_step": ms_step, "ms_per_step_stats": stats(t_wall),
        "tokens_per_s": tokens / (ms_step * 1e-3),
        "prefill": {"ms": pre["mean"], "ms_median": pre["median"], "ms_min": pre["min"],
                    "tokens_per_s": T / (pre["mean"] * 1e-3), "tflops": pre_flops / (pre["mean"] * 1e-3) / 1e12,
                    "frac_of_bf16_mfma_peak": pre_flops / (pre["mean"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF},
        "decode": {"ms": dec["mean"], "ms_median": dec["median"], "ms_min": dec["min"],
                   "ms_per_token_step": dec["mean"] / max(dsteps, 1), "tokens_per_s": batch * dsteps / max(dec["mean"] * 1e-3, 1e-9),
                   "gbytes_per_s": dec_bytes / max(dec["mean"] * 1e-3, 1e-9) / 1e9,
                   "frac_of_hbm_peak": dec_bytes / max(dec["mean"] * 1e-3, 1e-9) / 1e9 / HBM_PEAK_GBS},
    })
    if peaks:
        out["prefill"]["frac_of_measured_mfma_rate"] = out["prefill"]["tflops"] / out["measured_peaks"]["mfma_bf16_tflops"]
        out["decode"]["frac_of_measured_read_rate"] = out["decode"]["gbytes_per_s"] / out["measured_peaks"]["read_gbytes_per_s"]

    if probes:
        # prompt gate-up GEMM of one layer, probed in two more (untimed) prompt passes
        st.probe(B.LS_OP_GEMM_GATEUP, mid_layer, 0)
        st.prefill(x_prefill, lengths)
        st.prefill(x_prefill, lengths)
        torch.cuda.synchronize()
        probe_pre = st.probe_times()
        pre_exact = st.probe_is_kernel_exact()
        st.probe(B.LS_OP_NONE)
        timing = {True: "the kernel's own start/stop HIP events (stamped by the runtime at launch)",
                  False: "HIP events recorded around the operator's launches (includes launch gaps)"}
        d, F, e = shape.hidden, shape.ffn, shape.itemsize
        gu_bytes = 2 * F * d * e + batch * d * e + batch * F * e
        gu_ms = float(np.mean(probe_dec)) if probe_dec else float("nan")
        pg_flops = 2.0 * T * 2 * F * d
        pg_ms = float(np.mean(probe_pre)) if probe_pre else float("nan")
        out["probe_decode_gateup"] = {"bytes_per_launch": gu_bytes, "avg_ms": gu_ms, "launches_timed": len(probe_dec),
                                      "gbytes_per_s": gu_bytes / (gu_ms * 1e-3) / 1e9, "timing": timing[dec_exact]}
        out["probe_prefill_gateup"] = {"flops_per_launch": pg_flops, "avg_ms": pg_ms, "launches_timed": len(probe_pre),
                                       "tflops": pg_flops / (pg_ms * 1e-3) / 1e12, "timing": timing[pre_exact],
                                       "share_of_step": pg_ms * (hi - lo) / ms_step}
        out["probe_decode_gateup"]["share_of_step"] = gu_ms * (hi - lo) * dsteps / ms_step
    st.close()
    del st, x_prefill, x_decode, out_dec
    torch.cuda.empty_cache()
    return out, shape, lengths


def cpu_baseline(synth, shape, lo, hi, lengths, dsteps, budget_flop, threads):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the
    same workload: real layer dimensions and prompt lengths, but only as many layers (up to
    8), sequences and prompt rows as keep the work near `budget_flop` of fp64, and up to 8
    decode steps.  Throughput is per layer of the stage, scaled linearly to its layer count."""
    from oracle.stage_oracle import OracleStage

    import threadpoolctl

    p_mm = shape.qkv_rows * shape.hidden + shape.hidden * shape.n_q_heads * shape.head_dim + 3 * shape.ffn * shape.hidden
    L = hi - lo
    n_layers = min(L, 8)
    first = min(lengths[0], 1024)
    while n_layers > 1 and 2.0 * p_mm * n_layers * first > budget_flop:
        n_layers -= 1
    while first > 64 and 2.0 * p_mm * n_layers * first > budget_flop:
        first //= 2
    sample, tok = [first], first
    for n in lengths[1:]:
        if 2.0 * p_mm * n_layers * (tok + n) > budget_flop:
            break
        sample.append(n)
        tok += n
    n_seq = len(sample)
    n_dec = min(8, dsteps)
    one = shape.with_(vocab=0)
    mid = lo + (L - n_layers) // 2
    ora = OracleStage(one, mid, mid + n_layers, n_seq, max(sample) + n_dec)
    for l in range(mid, mid + n_layers):
        ora.load_tensors(l, synth.layer_tensors(one, SEED, l))
    x = synth.hidden_states(one, SEED + 1, sum(sample))
    xd = [synth.hidden_states(one, SEED + 2 + t, n_seq) for t in range(n_dec)]
    with threadpoolctl.threadpool_limits(limits=threads):
        t0 = time.perf_counter()
        ora.prefill(x, sample)
        for t in range(n_dec):
            ora.decode(xd[t])
        dt = time.perf_counter() - t0
        used = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] or [1])
    ntok = sum(sample) + n_seq * n_dec
    return {
        "value": ntok / (dt * L / n_layers), "unit": "tokens/s", "cores": used, "kind": "oracle",
        "sample": "%d of %d layers at real dims, %d of %d seqs (prompts of %s rows, %d decode steps each), %d tokens in %.1f s%s"
                  % (n_layers, L, n_seq, len(lengths), sorted(set(sample)), n_dec, ntok, dt,
                     "" if n_layers == L else "; scaled linearly to %d layers (extrapolated); embedding and LM head left out" % L),
    }


def execute_while_load(name, reps):
    """Time-to-first-token with the model streaming in from pinned host memory, against
    load-all-then-run, and the copy/compute overlap (per-block times from the library's own
    HIP events), then the workload's decode steps."""
    import torch

    import synth
    from paper_2502_09922_amd import Stage

    key, lo, hi, batch, prompt, dsteps = WORKLOADS[name]
    shape = synth.CONFIGS[key]
    lengths = [prompt] * batch
    T = batch * prompt
    st = Stage(shape, lo, hi, batch, prompt + dsteps, T)
    fill_blocks_on_device(st, SEED)
    ids = st.block_ids()
    # the model's home is pinned host memory: one packed block per layer (+ embedding, + head)
    blocks = {}
    for layer in ids:
        host = torch.empty(int(st_block_bytes(st, layer)), dtype=torch.uint8, pin_memory=True)
        host.copy_(st.block_view(layer))
        blocks[layer] = host
    torch.cuda.synchronize()
    st.slab.zero_()
    g = torch.Generator(device="cuda")
    g.manual_seed(SEED + 1)
    tok = torch.randint(0, shape.vocab, (T,), dtype=torch.int32, device="cuda", generator=g)
    copy = torch.cuda.Stream()
    st.set_profiling(True)

    def load_all(stream):
        st.reset_blocks()
        for layer in ids:
            st.load_block(layer, blocks[layer], stream=stream)

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3

    # warm-up (first-touch of pinned pages, kernel code load)
    load_all(copy); st.prefill(tok, lengths); torch.cuda.synchronize()
    runs = []
    for _ in range(max(1, reps)):
        # (1) copies alone: per-block copy time and completion time
        t_copy = timed(lambda: load_all(copy))
        c_end = {l: st.block_times(l)[1] for l in ids}
        c = {l: st.block_times(l)[0] for l in ids}
        # (2) prompt pass alone, everything resident: per-layer compute, embedding and head legs
        t_comp = timed(lambda: st.prefill(tok, lengths))
        p = st.layer_times(want_copy=False)["compute_ms"]
        p_before, p_after, _ = st.pass_times()
        # (3) load-all-then-run
        def serial():
            load_all(copy); torch.cuda.synchronize(); st.prefill(tok, lengths)
        t_serial = timed(serial)
        # (4) streamed: copies on the side stream, prompt pass gated per block
        def streamed():
            load_all(copy); return st.prefill(tok, lengths)
        t_stream = timed(streamed)
        lt = st.layer_times(want_copy=True)
        # ideal pipeline bound from the times measured alone: a block's work starts when the block
        # has landed and the work before it is done; the embedding gather and the head (final norm,
        # LM head, argmax) are stages of the recurrence like the layers
        f = max(0.0, c_end[ids[0]]) + p_before
        for i, l in enumerate(range(lo, hi)):
            f = max(f, c_end[l]) + p[i]
        f = max(f, c_end[ids[-1]]) + p_after
        sum_c, sum_p = sum(c.values()), sum(p) + p_before + p_after
        runs.append({
            "ttft_streamed_ms": t_stream, "ttft_load_all_then_run_ms": t_serial, "copy_alone_ms": t_copy,
            "prefill_alone_ms": t_comp, "sum_block_copy_ms": sum_c, "sum_compute_ms": sum_p,
            "ideal_pipeline_ms": f,
            "overlap_efficiency_E": (t_serial - t_stream) / max(t_serial - f, 1e-9),
            "copy_hidden_fraction_H": 1.0 - (t_stream - t_comp) / max(t_copy, 1e-9),
            "h2d_gbytes_per_s": sum(st_block_bytes(st, l) for l in ids) / (t_copy * 1e-3) / 1e9,
            "gate_ok": all(ce >= cp - 1e-3 for ce, cp in zip(lt["compute_end_ms"], lt["copy_end_ms"])),
        })
    best = dict(min(runs, key=lambda r: r["ttft_streamed_ms"]))
    # the decode steps that follow a streamed prompt pass (every block has landed: gates are no-ops)
    st.set_profiling(False)
    feed = streamed()
    torch.cuda.synchronize()
    outs = [torch.empty(batch, dtype=torch.int32, device="cuda") for _ in range(2)]
    t_dec = timed(lambda: [None for t in range(dsteps) for _ in [outs.__setitem__(t & 1, st.decode(feed if t == 0 else outs[(t - 1) & 1], batch, prompt + t, out=outs[t & 1]))]])
    best.update({"workload": name, "blocks": len(ids), "batch": batch, "prompt": prompt, "decode_steps": dsteps,
                 "decode_after_streamed_prefill_ms": t_dec, "decode_tokens_per_s": batch * dsteps / (t_dec * 1e-3),
                 "prompt_tokens_per_s_pcie_inclusive": T / (best["ttft_streamed_ms"] * 1e-3), "reps": len(runs)})
    st.close()
    del st, blocks
    torch.cuda.empty_cache()
    return best


def recorded_traffic(workload, key):
    """HBM bytes per launch of a kernel as measured by the rocprofv3 --pmc runs whose summary is
    committed under profiles/ (a profiler cannot run inside this script)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get(key)
    except (OSError, ValueError):
        return None


def device_info(torch):
    """What the run was measured on (name, compute units, memory; the library the timed calls ran in)."""
    p = torch.cuda.get_device_properties(0)
    import paper_2502_09922_amd.binding as B
    return {"name": p.name, "arch": getattr(p, "gcnArchName", ""), "compute_units": p.multi_processor_count,
            "hbm_bytes": p.total_memory, "library": os.path.relpath(B.LIB_PATH, ROOT)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default=DEFAULT, choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the other configurations (other_workloads, execute_while_load)")
    ap.add_argument("--decode-steps", type=int, default=None,
                    help="override the workload's number of decode steps (0: prompt pass only; for profiler runs)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch

    import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.workload.startswith("ewl_"):
        best = execute_while_load(args.workload, args.steps)
        print(json.dumps({
            "metric": "time-to-first-token, model streamed from pinned host memory (1 GPU)",
            "value": best["ttft_streamed_ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": 1,
            "ms_per_step": best["ttft_streamed_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic", "config": {"workload": args.workload}, "execute_while_load": best}))
        return

    if args.copy_probe:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    main_run, shape, lengths = run_throughput(args.workload, args.steps, args.warmup, probes=True, peaks=True,
                                              decode_steps=args.decode_steps)
    key, lo, hi, batch, prompt, dsteps = WORKLOADS[args.workload]
    if args.decode_steps is not None:
        dsteps = args.decode_steps
    if dsteps == 0:  # a profiler run of the prompt pass alone: phase numbers only
        print(json.dumps({"metric": "stage prefill tokens/s (1 GPU), prompt pass only", "value": main_run["prefill"]["tokens_per_s"],
                          "unit": "tokens/s", "config": {"workload": args.workload, "decode_steps": 0}, "prefill": main_run["prefill"]}))
        return
    pg, dg = main_run.pop("probe_prefill_gateup"), main_run.pop("probe_decode_gateup")
    # the kernel that takes the largest share of the step is the one `roofline` reports
    prefill_dominant = pg["share_of_step"] >= dg["share_of_step"]
    roof_pre = {"kernel": "prefill gate-up GEMM + SwiGLU", "bound": "mfma", "achieved": pg["tflops"],
                "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s", "frac": pg["tflops"] / MFMA_BF16_PEAK_TF,
                "traffic": recorded_traffic(args.workload, "prefill_gateup_gemm_bytes_per_launch"),
                "flops_per_launch": pg["flops_per_launch"], "avg_ms": pg["avg_ms"], "launches_timed": pg["launches_timed"],
                "share_of_step": pg["share_of_step"], "timing": pg["timing"]}
    roof_dec = {"kernel": "decode gate-up GEMM + SwiGLU", "bound": "hbm", "achieved": dg["gbytes_per_s"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": dg["gbytes_per_s"] / HBM_PEAK_GBS,
                "traffic": recorded_traffic(args.workload, "decode_gateup_gemm_bytes_per_launch"),
                "bytes_per_launch": dg["bytes_per_launch"], "avg_ms": dg["avg_ms"], "launches_timed": dg["launches_timed"],
                "share_of_step": dg["share_of_step"], "timing": dg["timing"]}
    res = {
        "metric": "stage prefill+decode tokens/s (1 GPU)",
        "value": main_run["tokens_per_s"],
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": main_run["ms_per_step"],
        "ms_per_step_median": main_run["ms_per_step_stats"]["median"],
        "ms_per_step_min": main_run["ms_per_step_stats"]["min"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if shape.dtype == "f32" else "bf16",
        "data": "synthetic",
        "device": device_info(torch),
        "config": {"workload": args.workload, "layers": [lo, hi], "batch": batch, "prompt": main_run["prompt"],
                   "decode_steps": dsteps, "embedding_and_lm_head": bool(shape.vocab), "vocab": shape.vocab,
                   "decode_feeds_back_its_tokens": main_run["feeds_back_tokens"], "setup_s": main_run["setup_s"],
                   "weights": "drawn on the device (torch generator, seed %d) into the slab, adopted as resident blocks" % SEED},
        "measured_peaks": main_run["measured_peaks"],
        "prefill": main_run["prefill"],
        "decode": main_run["decode"],
        "roofline": roof_pre if prefill_dominant else roof_dec,
        ("roofline_decode" if prefill_dominant else "roofline_prefill"): roof_dec if prefill_dominant else roof_pre,
    }
    if not args.no_extras and args.workload == DEFAULT:
        others = {}
        for name in EXTRAS:
            # each workload starts from an idle GPU: for some seconds after a long MFMA-heavy
            # pass the chip runs the bandwidth-bound decode kernels about 6 % slower
            time.sleep(IDLE_BEFORE_EXTRA_S)
            o, _, _ = run_throughput(name, 2 if "70b" in name else 5, 1, probes=False)
            o["idle_before_s"] = IDLE_BEFORE_EXTRA_S
            others[name] = {k: o[k] for k in ("layers", "batch", "prompt", "decode_steps", "steps", "warmup", "tokens_per_step",
                                              "ms_per_step", "tokens_per_s", "prefill", "decode", "idle_before_s")}
        res["other_workloads"] = others
        res["execute_while_load"] = execute_while_load(EWL, 3)
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(synth, shape, lo, hi, lengths, dsteps, 3e13, None)
        res["cpu_baseline_1_thread"] = cpu_baseline(synth, shape, lo, hi, lengths, dsteps, 2.5e12, 1)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
