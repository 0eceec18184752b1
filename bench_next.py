"""Measurements of the steps that follow the stage hot path, on one MI355X, synthetic data:

  --mode pipeline2d   two stages of a Llama-7B-shaped span on two streams, several
                      micro-batches in flight (Section 4.3) against the same calls issued one
                      after the other
  --mode kvrecompute  mode switch (Section 4.4): rebuilding a stage's KV cache by one prompt
                      pass over prompt + generated tokens, against copying the cache
  --mode blocks       block granularity on the host-to-device path (Section 7.6): the model
                      streamed as blocks of 1, 2, 4, 8 layers and as one block; one copy per
                      tensor and two per layer instead of one per packed block (tensor packing,
                      Section 5); a fresh device allocation per block instead of the slab
                      allocated up front (GPU memory pre-allocation, Section 5)

Each mode prints ONE JSON line.  Weights are seeded N(0, 0.02) as in bench.py.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import bench  # noqa: E402  (stage construction and seeds are shared with the main benchmark)

SEED = bench.SEED


def dev(torch, a):
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def wall_ms(torch, fn, reps):
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(reps):
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        best = min(best, (time.perf_counter() - t0) * 1e3)
    return best


def pipeline2d(args):
    import torch
    import synth
    from paper_2502_09922_amd import MicroBatch, Pipeline, Stage, pack_block

    shape = synth.CONFIGS["llama7b"].with_(vocab=0)
    lo, mid, hi = 8, 12, 16
    n_micro, mb_batch, prompt, dsteps = 4, 2, 512, 32
    lengths = [prompt] * mb_batch
    stages = []
    for a, b in ((lo, mid), (mid, hi)):
        st, blocks = bench.build_stage(synth, Stage, pack_block, shape, a, b, lengths, dsteps)
        for layer in st.block_ids():
            st.load_block(layer, blocks[layer])
        stages.append(st)
    torch.cuda.synchronize()
    pipe = Pipeline(stages)
    mbs = [MicroBatch(pipe, mb_batch * prompt) for _ in range(n_micro)]
    x_pre = [dev(torch, synth.hidden_states(shape, SEED + 1 + m, mb_batch * prompt)) for m in range(n_micro)]
    x_dec = [[dev(torch, synth.hidden_states(shape, SEED + 100 + 7 * m + t, mb_batch)) for m in range(n_micro)]
             for t in range(dsteps)]

    def reset():
        for mb in mbs:
            for _, _, sl in mb.caches:
                sl.zero_()

    def pipelined():
        reset()
        pipe.run(0, mbs, x_pre, lengths=[lengths] * n_micro)
        for t in range(dsteps):
            pipe.run(1, mbs, x_dec[t], max_ctx=[prompt + t] * n_micro)

    def serial():
        # the same calls, but each waits for the one before it (no two in flight)
        reset()
        for m in range(n_micro):
            pipe.run(0, [mbs[m]], [x_pre[m]], lengths=[lengths])
            torch.cuda.synchronize()
        for t in range(dsteps):
            for m in range(n_micro):
                pipe.run(1, [mbs[m]], [x_dec[t][m]], max_ctx=[prompt + t])
                torch.cuda.synchronize()

    pipelined(); serial()
    t_pipe = wall_ms(torch, pipelined, args.steps)
    t_ser = wall_ms(torch, serial, args.steps)
    tokens = n_micro * mb_batch * (prompt + dsteps)
    out = {
        "metric": "2-stage pipeline, 4 micro-batches in flight: tokens/s (1 GPU)", "value": tokens / (t_pipe * 1e-3),
        "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": 1, "ms_per_step": t_pipe,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "pipe2d_llama7b_l8_12_16_mb4x2_s512_d32", "stages": [[lo, mid], [mid, hi]],
                   "micro_batches": n_micro, "batch_per_micro_batch": mb_batch, "prompt": prompt, "decode_steps": dsteps},
        "pipeline2d": {"pipelined_ms": t_pipe, "one_call_at_a_time_ms": t_ser, "speedup": t_ser / t_pipe,
                       "note": "both stages share one GPU: the gain is what overlapping two streams hides of "
                               "launch gaps and kernel tails, not a second device's throughput"},
    }
    print(json.dumps(out))
    pipe.close()
    for st in stages:
        st.close()


def kvrecompute(args):
    import torch
    import synth
    from paper_2502_09922_amd import Stage, pack_block

    shape = synth.CONFIGS["llama7b"].with_(vocab=0)
    lo, hi, batch, prompt, gen = 8, 16, 8, 512, 128
    new_len = [prompt + gen] * batch
    st, blocks = bench.build_stage(synth, Stage, pack_block, shape, lo, hi, new_len, 1)
    for layer in st.block_ids():
        st.load_block(layer, blocks[layer])
    x = dev(torch, synth.hidden_states(shape, SEED + 1, sum(new_len)))
    torch.cuda.synchronize()
    st.prefill(x, new_len)
    t_re = wall_ms(torch, lambda: st.prefill(x, new_len), args.steps)
    # the alternative: move the cache.  Bytes that hold live positions, both K and V.
    e = shape.itemsize
    live = (hi - lo) * batch * shape.n_kv_heads * (prompt + gen) * shape.head_dim * e * 2
    k2, v2 = torch.empty_like(st.k), torch.empty_like(st.v)
    t_d2d = wall_ms(torch, lambda: (k2.copy_(st.k), v2.copy_(st.v)), args.steps)
    hk = torch.empty(st.k.numel(), dtype=torch.uint8, pin_memory=True)
    hv = torch.empty(st.v.numel(), dtype=torch.uint8, pin_memory=True)
    hk.copy_(st.k); hv.copy_(st.v)
    t_h2d = wall_ms(torch, lambda: (k2.copy_(hk, non_blocking=True), v2.copy_(hv, non_blocking=True)), args.steps)
    alloc = 2 * st.k.numel()
    out = {
        "metric": "KV-cache recomputation time on mode switch (1 GPU)", "value": t_re, "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": 1, "ms_per_step": t_re, "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "kvrecompute_llama7b_l8_16_b8_s512_g128", "layers": [lo, hi], "batch": batch,
                   "prompt": prompt, "generated": gen},
        "kv_recompute": {"recompute_ms": t_re, "tokens_recomputed": sum(new_len),
                         "cache_bytes_live": live, "cache_bytes_allocated": alloc,
                         "copy_device_to_device_ms": t_d2d, "copy_from_pinned_host_ms": t_h2d,
                         "host_link_gbytes_per_s": alloc / (t_h2d * 1e-3) / 1e9,
                         "note": "the paper recomputes because moving caches between nodes needs all-to-all "
                                 "traffic over the network; on one GPU the copy legs above are the local bounds"},
    }
    print(json.dumps(out))
    st.close()


def blocks_mode(args):
    import torch
    import synth
    from paper_2502_09922_amd import Stage, pack_block, binding as B

    shape = synth.CONFIGS["llama7b"].with_(vocab=0)
    lo, hi, batch, prompt = 0, 32, 16, 512
    lengths = [prompt] * batch
    st, blocks = bench.build_stage(synth, Stage, pack_block, shape, lo, hi, lengths, 1)
    # one pinned buffer with all layer blocks back to back (what a coarser block looks like)
    per = blocks[lo].numel()
    big = torch.empty(per * (hi - lo), dtype=torch.uint8, pin_memory=True)
    for l in range(lo, hi):
        big[(l - lo) * per:(l - lo + 1) * per].copy_(blocks[l])
    x = dev(torch, synth.hidden_states(shape, SEED + 1, batch * prompt))
    copy = torch.cuda.Stream()
    for layer in st.block_ids():
        st.load_block(layer, blocks[layer])
    st.prefill(x, lengths)
    torch.cuda.synchronize()
    t_compute = wall_ms(torch, lambda: st.prefill(x, lengths), args.steps)
    rows = []
    for g in (1, 2, 4, 8, 16, 32):
        def load():
            st.reset_blocks()
            for l in range(lo, hi, g):
                st.load_layers(l, l + g - 1, big[(l - lo) * per:(l - lo + g) * per], stream=copy)
        def streamed():
            load()
            st.prefill(x, lengths)
        streamed()
        rows.append({"layers_per_block": g, "blocks": (hi - lo) // g, "copy_alone_ms": wall_ms(torch, load, args.steps),
                     "ttft_streamed_ms": wall_ms(torch, streamed, args.steps)})
    # tensor packing: six copies per layer (one per tensor) instead of one per packed block
    cfg = st.cfg
    spans = []
    off, nb = B.C.c_size_t(), B.C.c_size_t()
    for i in range(6):
        B.check(B.ls_block_tensor(B.C.byref(cfg), lo, i, B.C.byref(off), B.C.byref(nb)))
        spans.append((off.value, nb.value))
    slab = st.slab
    def per_tensor():
        with torch.cuda.stream(copy):
            for l in range(lo, hi):
                base = (l - lo) * per
                for o, n in spans:
                    slab[base + o: base + o + n].copy_(big[base + o: base + o + n], non_blocking=True)
    per_tensor()
    t_tensor = wall_ms(torch, per_tensor, args.steps)
    # half-layer blocks: the attention tensors and the FFN tensors of a layer as two copies
    half = spans[3][0]  # offset of the FFN norm gain = end of the attention half
    def half_layer():
        with torch.cuda.stream(copy):
            for l in range(lo, hi):
                base = (l - lo) * per
                slab[base: base + half].copy_(big[base: base + half], non_blocking=True)
                slab[base + half: base + per].copy_(big[base + half: base + per], non_blocking=True)
    half_layer()
    t_half = wall_ms(torch, half_layer, args.steps)
    # allocate on arrival: a fresh device allocation per block (hipMalloc, then the copy, freed
    # afterwards) instead of the slab allocated once up front (Section 5, GPU memory pre-allocation)
    hip = B.C.CDLL("libamdhip64.so")
    hip.hipMalloc.argtypes = [B.C.POINTER(B.C.c_void_p), B.C.c_size_t]
    hip.hipFree.argtypes = [B.C.c_void_p]
    hip.hipMemcpyAsync.argtypes = [B.C.c_void_p, B.C.c_void_p, B.C.c_size_t, B.C.c_int, B.C.c_void_p]
    def alloc_on_arrival():
        ptrs = []
        for l in range(lo, hi):
            ptr = B.C.c_void_p()
            assert hip.hipMalloc(B.C.byref(ptr), per) == 0
            assert hip.hipMemcpyAsync(ptr, big.data_ptr() + (l - lo) * per, per, 1, copy.cuda_stream) == 0
            ptrs.append(ptr)
        copy.synchronize()
        return ptrs
    def alloc_run():
        for ptr in alloc_on_arrival():
            assert hip.hipFree(ptr) == 0
    alloc_run()
    t_alloc = wall_ms(torch, alloc_run, args.steps)
    best = min(rows, key=lambda r: r["ttft_streamed_ms"])
    out = {
        "metric": "time-to-first-token by block granularity, model streamed from pinned host memory (1 GPU)",
        "value": best["ttft_streamed_ms"], "unit": "ms", "n_gpus": 1, "steps": args.steps, "warmup": 1,
        "ms_per_step": best["ttft_streamed_ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "blocks_llama7b_32layers_b16_s512", "batch": batch, "prompt": prompt,
                   "model_bytes": per * (hi - lo)},
        "block_granularity": {"prefill_alone_ms": t_compute, "sweep": rows,
                              "copy_one_per_tensor_ms": t_tensor,
                              "copy_two_per_layer_ms": t_half,
                              "copy_one_per_packed_block_ms": rows[0]["copy_alone_ms"],
                              "copy_into_fresh_allocation_per_block_ms": t_alloc,
                              "note": "the fresh-allocation figure includes the 32 hipMalloc and hipFree calls"},
    }
    print(json.dumps(out))
    st.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mode", required=True, choices=["pipeline2d", "kvrecompute", "blocks"])
    ap.add_argument("--steps", type=int, default=3)
    args = ap.parse_args()
    import torch

    assert torch.cuda.is_available(), "bench_next.py needs a GPU"
    {"pipeline2d": pipeline2d, "kvrecompute": kvrecompute, "blocks": blocks_mode}[args.mode](args)


if __name__ == "__main__":
    main()
