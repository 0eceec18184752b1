"""Benchmark of the stage hot path on one MI355X.

One step = one pass of the whole hot path over one batch: the prompt pass of the stage
followed by the KV-cached decode steps of the workload.  Default workload: the
Llama-7B-shaped middle stage (layers 8..15 of 32, bf16), batch 8 x 512 prompt tokens of
N(0,1) hidden states, then 128 decode steps.  Weights are seeded synthetic N(0, 0.02)
(gains 1 + N(0, 0.02)), packed per layer, copied from pinned host memory by the library's
loader and resident in HBM before the timed region starts.

Prints ONE JSON line (see the keys below).  `value` is tokens handled per second over the
whole step (prompt tokens + generated tokens, divided by prefill + decode time).
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
    "llama7b_stage_l8_16_b8_s512_d128": ("llama7b", 8, 16, 8, 512, 128),
    "tiny_f32_b1_s32_d8": ("tiny_f32", 0, 2, 1, 32, 8),
    # slices of the larger benchmark configurations (fewer layers, same per-layer shapes)
    "llama13b_l4_b32_s1024_d16": ("llama13b", 16, 20, 32, 1024, 16),
    "llama70b_l4_b64_ragged128_2048_d16": ("llama70b", 40, 44, 64, (128, 2048), 16),
    # execute-while-load: the whole 7B-shaped model streams in as 34 blocks while prefill runs
    "ewl_llama7b_full_b16_s512_d32": ("llama7b", 0, 32, 16, 512, 32),
    # same model, a prompt batch heavy enough that compute, not the host link, is the longer leg
    "ewl_llama7b_full_b64_s512_d32": ("llama7b", 0, 32, 64, 512, 32),
}
SEED = 1234


def prompt_lengths(synth, batch, prompt):
    """Uniform prompts, or (lo, hi): seeded ragged lengths uniform on [lo, hi]."""
    if isinstance(prompt, tuple):
        return [int(n) for n in synth.ragged_lengths(SEED + 7, batch, prompt[0], prompt[1])]
    return [prompt] * batch


def build_stage(synth, Stage, pack_block, shape, lo, hi, lengths, steps):
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


def st_block_bytes(st, layer):
    from paper_2502_09922_amd import binding as b

    return b.ls_stage_block_bytes(st.handle, layer)


def cpu_baseline(synth, shape, lo, hi, lengths, dsteps):
    """The oracle as it stands, timed on this machine's host cores on a bounded sample of the
    same workload: real layer dimensions and prompt lengths, but only as many layers (up to
    8) and sequences as keep the work near 15 TFLOP of fp64 (about 15-30 s here), and 8
    decode steps.  Throughput is per layer of the stage, scaled linearly to its layer count."""
    from oracle.stage_oracle import OracleStage

    import threadpoolctl

    p_mm = shape.qkv_rows * shape.hidden + shape.hidden * shape.n_q_heads * shape.head_dim + 3 * shape.ffn * shape.hidden
    budget = 15e12
    n_layers = min(hi - lo, 8)
    while n_layers > 1 and 2.0 * p_mm * n_layers * lengths[0] > budget:
        n_layers -= 1
    n_seq, tok = 0, 0
    while n_seq < len(lengths) and (n_seq == 0 or 2.0 * p_mm * n_layers * (tok + lengths[n_seq]) <= budget):
        tok += lengths[n_seq]
        n_seq += 1
    sample = list(lengths[:n_seq])
    n_dec = min(8, dsteps)
    one = shape.with_(vocab=0)
    ora = OracleStage(one, lo, lo + n_layers, n_seq, max(sample) + n_dec)
    for l in range(lo, lo + n_layers):
        ora.load_tensors(l, synth.layer_tensors(one, SEED, l))
    x = synth.hidden_states(one, SEED + 1, sum(sample))
    t0 = time.perf_counter()
    ora.prefill(x, sample)
    for t in range(n_dec):
        ora.decode(synth.hidden_states(one, SEED + 2 + t, n_seq))
    dt = time.perf_counter() - t0
    threads = max([p["num_threads"] for p in threadpoolctl.threadpool_info()] or [1])
    return dt, sum(sample) + n_seq * n_dec, threads, n_layers, n_dec, n_seq, max(sample)


def execute_while_load(args, synth, st, blocks, shape, batch, prompt, dsteps):
    """Time-to-first-token with the model streaming in from pinned host memory, against
    load-all-then-run, and the copy/compute overlap (per-layer times from the library's
    own HIP events)."""
    import torch

    T = batch * prompt
    tok = torch.from_numpy(synth.token_ids(SEED + 1, T, shape.vocab)).cuda()
    lengths = [prompt] * batch
    compute = torch.cuda.current_stream()
    copy = torch.cuda.Stream()
    ids = st.block_ids()
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
    res = {"runs": []}
    for _ in range(max(1, args.steps)):
        # (1) copies alone
        t_copy = timed(lambda: load_all(copy))
        lt_c = st.layer_times(want_copy=True)
        c, c_end = lt_c["copy_ms"], lt_c["copy_end_ms"]
        # (2) prompt pass alone, everything resident
        t_comp = timed(lambda: st.prefill(tok, lengths))
        p = st.layer_times(want_copy=True)["compute_ms"]
        # (3) load-all-then-run
        def serial():
            load_all(copy); torch.cuda.synchronize(); st.prefill(tok, lengths)
        t_serial = timed(serial)
        # (4) streamed: copies on the side stream, prompt pass gated per layer
        def streamed():
            load_all(copy); st.prefill(tok, lengths)
        t_stream = timed(streamed)
        lt = st.layer_times(want_copy=True)
        # ideal pipeline bound from the per-layer times measured alone: a layer starts when
        # its block has landed and the previous layer is done; the head follows the last layer
        f = 0.0
        for ce, pi in zip(c_end, p):
            f = max(f, ce) + pi
        sum_c, sum_p = sum(c), sum(p)
        f = max(f, t_copy) + max(t_comp - sum_p, 0.0) * 0.5
        res["runs"].append({
            "ttft_streamed_ms": t_stream, "ttft_load_all_then_run_ms": t_serial, "copy_alone_ms": t_copy,
            "prefill_alone_ms": t_comp, "sum_layer_copy_ms": sum_c, "sum_layer_compute_ms": sum_p,
            "ideal_pipeline_ms": f,
            "overlap_efficiency_E": (t_serial - t_stream) / max(t_serial - f, 1e-9),
            "copy_hidden_fraction_H": 1.0 - (t_stream - t_comp) / max(t_copy, 1e-9),
            "h2d_gbytes_per_s": sum(st_block_bytes(st, l) for l in ids) / (t_copy * 1e-3) / 1e9,
            "gate_ok": all(ce >= cp - 1e-3 for ce, cp in zip(lt["compute_end_ms"], lt["copy_end_ms"])),
        })
    best = min(res["runs"], key=lambda r: r["ttft_streamed_ms"])
    out = {
        "metric": "time-to-first-token, model streamed from pinned host memory (1 GPU)",
        "value": best["ttft_streamed_ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": 1,
        "ms_per_step": best["ttft_streamed_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": args.workload, "blocks": len(ids), "batch": batch, "prompt": prompt},
        "execute_while_load": best,
    }
    print(json.dumps(out))


def recorded_traffic(workload):
    """HBM bytes per launch of the dominant kernel as measured by the rocprofv3 --pmc runs
    whose summary is committed under profiles/ (a profiler cannot run inside this script)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(workload, {}).get("decode_gateup_gemm_bytes_per_launch")
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
    ap.add_argument("--workload", default="llama7b_stage_l8_16_b8_s512_d128", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 1 GiB device copy (calibrates rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch

    import synth
    from paper_2502_09922_amd import Stage, pack_block, binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    key, lo, hi, batch, prompt, dsteps = WORKLOADS[args.workload]
    shape = synth.CONFIGS[key]
    t_gen = time.perf_counter()
    lengths = prompt_lengths(synth, batch, prompt)
    max_len = max(lengths)
    st, blocks = build_stage(synth, Stage, pack_block, shape, lo, hi, lengths, dsteps)
    t_gen = time.perf_counter() - t_gen
    if args.workload.startswith("ewl_"):
        execute_while_load(args, synth, st, blocks, shape, batch, prompt, dsteps)
        st.close()
        return
    stream = torch.cuda.current_stream()
    for layer in st.block_ids():
        st.load_block(layer, blocks[layer], stream=stream)
    torch.cuda.synchronize()

    if args.copy_probe:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # what this GPU sustains for the two bounding resources (outside the timed region): the
    # resident weight slab read once with the decode kernels' loads, and a register-only MFMA loop
    import ctypes
    cur = ctypes.c_void_p(stream.cuda_stream)
    sink = torch.zeros(4, dtype=torch.float32, device="cuda")
    peak_read = B.ls_probe_read_gbps(ctypes.c_void_p(st.slab.data_ptr()), st.slab.numel(), 3,
                                     ctypes.c_void_p(sink.data_ptr()), cur)
    peak_mfma = B.ls_probe_mfma_tflops(2000, 3, ctypes.c_void_p(sink.data_ptr()), cur)
    assert peak_read > 0 and peak_mfma > 0, B.ls_last_error()

    T = sum(lengths)
    if st.first:
        x_prefill = torch.from_numpy(synth.token_ids(SEED + 1, T, shape.vocab)).cuda()
        x_decode = [torch.from_numpy(synth.token_ids(SEED + 2 + t, batch, shape.vocab)).cuda() for t in range(dsteps)]
    else:
        def dev(a):
            if a.dtype == np.uint16:
                return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
            return torch.from_numpy(a).cuda()
        x_prefill = dev(synth.hidden_states(shape, SEED + 1, T))
        x_decode = [dev(synth.hidden_states(shape, SEED + 2 + t, batch)) for t in range(dsteps)]
    out_dec = (torch.empty(batch, dtype=torch.int32, device="cuda") if st.last
               else torch.empty(batch, shape.hidden, dtype=st.tdtype, device="cuda"))
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    mid_layer = (lo + hi) // 2
    PROBED = min(16, dsteps)  # decode steps per step whose gate-up launch is probed
    probe_lo = (dsteps - PROBED) // 2
    probe_hi = probe_lo + PROBED

    def one_step(timed):
        if timed:
            ev[0].record(stream)
        st.prefill(x_prefill, lengths)
        if timed:
            ev[1].record(stream)
        for t in range(dsteps):
            # the probe (runtime-stamped start/stop events on one layer's gate-up launch) costs
            # a few microseconds per probed launch: it is on for PROBED decode steps of a step
            if timed and t == probe_lo:
                st.probe(B.LS_OP_GEMM_GATEUP, mid_layer, 1)
            if timed and t == probe_hi:
                st.probe(B.LS_OP_NONE)
            st.decode(x_decode[t], batch, max_len + t, out=out_dec)
        if timed:
            ev[2].record(stream)

    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()

    # the decode gate-up GEMM (the kernel that moves the most bytes) of one layer is probed
    # inside the timed region, see one_step
    t_pre = t_dec = 0.0
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    probe_dec, dec_exact = [], True
    for _ in range(args.steps):
        one_step(True)
        torch.cuda.synchronize()
        t_pre += ev[0].elapsed_time(ev[1])
        t_dec += ev[1].elapsed_time(ev[2])
        probe_dec.extend(st.probe_times())
        dec_exact = dec_exact and st.probe_is_kernel_exact()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    st.probe(B.LS_OP_NONE)

    # one more (untimed) prompt pass with the probe on the prefill gate-up GEMM
    st.probe(B.LS_OP_GEMM_GATEUP, mid_layer, 0)
    st.prefill(x_prefill, lengths)
    st.prefill(x_prefill, lengths)
    torch.cuda.synchronize()
    probe_pre = st.probe_times()
    pre_exact = st.probe_is_kernel_exact()
    st.probe(B.LS_OP_NONE)
    timing = {True: "the kernel's own start/stop HIP events (stamped by the runtime at launch)",
              False: "HIP events recorded around the operator's launches (includes launch gaps)"}

    ms_step = wall * 1e3 / args.steps
    t_pre /= args.steps
    t_dec /= args.steps
    tokens = T + batch * dsteps
    d, F, e = shape.hidden, shape.ffn, shape.itemsize
    # decode gate-up GEMM: algorithmic bytes = the two stacked projections read once, plus
    # the activations in and out
    gu_bytes = 2 * F * d * e + batch * d * e + batch * F * e
    gu_ms = float(np.mean(probe_dec)) if probe_dec else float("nan")
    achieved = gu_bytes / (gu_ms * 1e-3) / 1e9
    # prefill gate-up GEMM: 2 * T * 2F * d flops
    pg_flops = 2.0 * T * 2 * F * d
    pg_ms = float(np.mean(probe_pre)) if probe_pre else float("nan")
    pg_tf = pg_flops / (pg_ms * 1e-3) / 1e12

    # whole-phase algorithmic work
    L = hi - lo
    wbytes = sum(st_block_bytes(st, l) for l in range(lo, hi))
    kv_tok = 2 * shape.n_kv_heads * shape.head_dim * e
    dec_bytes = sum(wbytes + (T + batch * (t + 1)) * kv_tok * L for t in range(dsteps))
    p_mm = (shape.qkv_rows * d + d * shape.n_q_heads * shape.head_dim + 3 * F * d)
    pre_flops = 2.0 * T * p_mm * L + sum(2.0 * shape.n_q_heads * shape.head_dim * n * (n + 1) for n in lengths) * L

    res = {
        "metric": "stage prefill+decode tokens/s (1 GPU)",
        "value": tokens / (ms_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32" if shape.dtype == "f32" else "bf16",
        "data": "synthetic",
        "device": device_info(torch),
        "config": {"workload": args.workload, "layers": [lo, hi], "batch": batch,
                   "prompt": prompt if isinstance(prompt, int) else {"ragged": list(prompt), "total_tokens": T},
                   "decode_steps": dsteps, "weights_gen_s": round(t_gen, 1)},
        "measured_peaks": {"read_gbytes_per_s": peak_read, "mfma_bf16_tflops": peak_mfma,
                           "how": "ls_probe_read_gbps over the resident weight slab, ls_probe_mfma_tflops (register-only loop)"},
        "prefill": {"ms": t_pre, "tokens_per_s": T / (t_pre * 1e-3), "tflops": pre_flops / (t_pre * 1e-3) / 1e12,
                    "frac_of_bf16_mfma_peak": pre_flops / (t_pre * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF,
                    "frac_of_measured_mfma_rate": pre_flops / (t_pre * 1e-3) / 1e12 / peak_mfma},
        "decode": {"ms": t_dec, "ms_per_token_step": t_dec / dsteps, "tokens_per_s": batch * dsteps / (t_dec * 1e-3),
                   "gbytes_per_s": dec_bytes / (t_dec * 1e-3) / 1e9,
                   "frac_of_hbm_peak": dec_bytes / (t_dec * 1e-3) / 1e9 / HBM_PEAK_GBS,
                   "frac_of_measured_read_rate": dec_bytes / (t_dec * 1e-3) / 1e9 / peak_read},
        "roofline": {"kernel": "decode gate-up GEMM + SwiGLU", "bound": "hbm", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": recorded_traffic(args.workload),
                     "bytes_per_launch": gu_bytes, "avg_ms": gu_ms, "launches_timed": len(probe_dec),
                     "timing": timing[dec_exact]},
        "roofline_prefill": {"kernel": "prefill gate-up GEMM + SwiGLU", "bound": "mfma", "achieved": pg_tf,
                             "peak": MFMA_BF16_PEAK_TF, "unit": "TFLOP/s", "frac": pg_tf / MFMA_BF16_PEAK_TF,
                             "flops_per_launch": pg_flops, "avg_ms": pg_ms, "launches_timed": len(probe_pre),
                             "timing": timing[pre_exact]},
    }
    if not args.no_cpu_baseline:
        dt, ntok, threads, n_layers, n_dec, n_seq, s_max = cpu_baseline(synth, shape, lo, hi, lengths, dsteps)
        res["cpu_baseline"] = {
            "value": ntok / (dt * L / n_layers), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d of %d layers at real dims, %d of %d seqs (prompts up to %d, %d decode steps each), "
                      "%d tokens in %.1f s%s"
                      % (n_layers, L, n_seq, batch, s_max, n_dec, ntok, dt,
                         "" if n_layers == L else "; scaled linearly to %d layers (extrapolated)" % L),
        }
    st.close()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
