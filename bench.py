"""Benchmark of the compressed-shard hot path on one MI355X.

A step is one pass of a 70B-shaped shard layer over one prefill batch of 4096 tokens (the largest of the
workloads): the incoming hidden state [4096, 8192] is decoded from its blockwise 8-bit form (inside the first
linear's preparation kernel), the four linears of the decoder layer (QKV 8192->10240, O 8192->8192, gate/up
8192->57344, down 28672->8192) run through the mixed int8 decomposition (outlier scan + row absmax + int8
codes, int8 MFMA GEMM with the fused epilogue), and the outgoing hidden state (the last linear's output plus
the residual stream) is encoded again in that linear's epilogue.  Weights are pre-quantized before the timed
region (they are static).  Inputs are seeded synthetic tensors drawn on the host by the workload recipes and
resident in HBM when the timed region starts.  Prints one JSON line; further sections of that line hold the
Llama-7B-shaped shard (2048 tokens, 4 layers) as a second timed step, the codec alone on the [8192, 8192]
boundary state, the decode shapes and the companions of the layer.
"""
import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0      # MI355X dense int8 MFMA, TOP/s
HBM_PEAK_GBS = 8000.0
# What the matrix pipes alone sustain on this kind of data within the package power limit: a register-only
# v_mfma_i32_32x32x32_i8 loop on Gaussian int8 codes, eight waves per CU (profiles/mfma_i8_power_ceiling.txt).
INT8_POWER_LIMITED_TOPS = 3468.0
# HBM bytes per GEMM launch (mean over the five launches of a decoder layer) from rocprofv3 FETCH_SIZE and
# WRITE_SIZE, each scaled by what the same counter reads for kernels of known traffic in the same runs
# (profiles/gemm_llama70b_prefill_counters.txt, profiles/gemm_llama7b_prefill_counters.txt): the timed step
# (70B-shaped layer, 4096 tokens) and the 7B-shaped step.  Valid for the GEMM source they were measured on:
# reported as null once that file has changed.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 1185.3e6
GEMM_TRAFFIC_BYTES_PER_LAUNCH_7B = 182.6e6
GEMM_TRAFFIC_SOURCE_SHA256 = "d31feb445e95096b1c0fff96f120c4d970f74e19a65f82518998941645101b22"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=4, help="decoder layers of the 7B-shaped second step")
    ap.add_argument("--codec-block", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--sections", default="all",
                    help="profiling aid: comma-separated sections to run instead of all of them: step (the 70B-shaped "
                         "timed step), 7b (the 7B-shaped timed step), codec, decode, heavy, readings, adapter, exit, vit, "
                         "prequant, kv")
    ap.add_argument("--gemm-tiles", type=int, default=-1, help="tuning: force a GEMM tile configuration (-1 = automatic)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (a kernel of known HBM traffic, to scale rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    return ap.parse_args()


class HipEvents:
    """hipEvent_t handles made through the HIP runtime, so that the library can record them."""

    def __init__(self):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self):
        ev = ctypes.c_void_p()
        assert self.hip.hipEventCreate(ctypes.byref(ev)) == 0
        return ev.value

    def quad(self):
        """(begin, gemm_begin, gemm_end, prep_mid) as the binding takes them."""
        return [self.create() for _ in range(4)]

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value


def gemm_traffic(value=None):
    import hashlib
    src = os.path.join(ROOT, "paper_2407_19775_amd", "csrc", "gemm_kernels.hip")
    try:
        same = hashlib.sha256(open(src, "rb").read()).hexdigest() == GEMM_TRAFFIC_SOURCE_SHA256
    except OSError:
        same = False
    return (GEMM_TRAFFIC_BYTES_PER_LAUNCH if value is None else value) if same else None


def cpu_baseline(sample, hidden, block):
    """The CPU oracle, as it stands, on one step's worth of work: the layer's four linears at full size (all 4096
    tokens) plus one codec round trip of the [4096, 8192] hidden state with the step's block size (10-15 s on 16
    cores).  sample: list of (name, X, W) host arrays."""
    from oracle import blockwise_codec as bc
    from oracle import mixed_linear as ml
    from paper_2407_19775_amd import workloads as wl
    prepared, ops = [], 0
    for _, X, W in sample:
        Wq, c = ml.prequantize_weight(W)             # offline step, untimed like on the GPU
        prepared.append((X, Wq, c))
        ops += 2 * X.shape[0] * W.shape[0] * W.shape[1]
    t0 = time.perf_counter()
    codes, a = bc.quantize_blockwise(hidden, block)
    bc.dequantize_blockwise(codes, a, block)
    for X, Wq, c in prepared:
        ml.mixed_int8_linear(X, Wq, c, wl.TAU)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": "the %s linears of the step at full size (4096 tokens, %.2f of its 7.01 TOP) + one codec round trip "
                      "of the [4096,8192] hidden state, block %d; %.1f s" % ("/".join(n for n, _, _ in sample), ops / 1e12, block, dt)}


def timed_wall(step, steps, warmup, torch):
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def events_pass(step, evs, reps, he, torch):
    """Mean per-call times from the library's events: (whole preparation, its first kernel, GEMM kernel), ms."""
    n = len(evs)
    prep, prep1, gemm = [0.0] * n, [0.0] * n, [0.0] * n
    for _ in range(reps):
        step(evs)
        torch.cuda.synchronize()
        for i, (e0, e1, e2, em) in enumerate(evs):
            prep[i] += he.elapsed_ms(e0, e1) / reps
            prep1[i] += he.elapsed_ms(e0, em) / reps
            gemm[i] += he.elapsed_ms(e1, e2) / reps
    return prep, prep1, gemm


def linear_row(M, shp, gemm_ms, prep_ms, prep1_ms):
    ops = 2.0 * M * shp.K * shp.N
    bytes3 = 3.0 * M * shp.K
    return {"gemm_us": round(gemm_ms * 1e3, 1), "gemm_tops": round(ops / gemm_ms / 1e9, 1),
            "pct_int8_peak": round(100.0 * ops / gemm_ms / 1e9 / INT8_PEAK_TOPS, 1),
            "prep_us": round(prep_ms * 1e3, 1), "prep_gbs": round(bytes3 / prep_ms / 1e6, 1),
            "prep_pct_hbm": round(100.0 * bytes3 / prep_ms / 1e6 / HBM_PEAK_GBS, 1),
            "scan_pack_us": round(prep1_ms * 1e3, 1), "scan_pack_gbs": round(bytes3 / prep1_ms / 1e6, 1),
            "scan_pack_pct_hbm": round(100.0 * bytes3 / prep1_ms / 1e6 / HBM_PEAK_GBS, 1)}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures one GPU: this library has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    from paper_2407_19775_amd import binding, workloads as wl

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    tune = binding.tune_gemm_tiles(args.gemm_tiles) if args.gemm_tiles >= 0 else 0
    chosen = set(args.sections.split(","))

    def want(name):
        return "all" in chosen or name in chosen

    block = args.codec_block
    he = HipEvents()
    out = {}

    def timed(fn, n=20):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fn()
        fn()
        a.record()
        for _ in range(n):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / n

    # =================================================================== the step: 70B-shaped layer, 4096 tokens
    cpu_sample, hidden_host = [], None
    if want("step"):
        M5, shapes5 = 4096, wl.LLAMA_70B_LINEARS
        X5h = {K: wl.prefill_activation(5, 10 + K % 5, M5, K)[0] for K in sorted({s.K for s in shapes5})}
        X5 = {K: torch.from_numpy(x).to(dev) for K, x in X5h.items()}
        w5 = []
        for i, shp in enumerate(shapes5):
            Wh = wl.prefill_weight(5, 20 + i, shp, 0.015)
            W = torch.from_numpy(Wh).to(dev)
            w5.append(binding.prequantize_weight(W))
            del W
            if not args.no_cpu_baseline:
                cpu_sample.append((shp.name, X5h[shp.K], Wh))          # the oracle's sample: the step's own tensors
            del Wh
        hidden_host = X5h[8192]
        Y5 = {s.name: torch.empty((M5, s.N), dtype=torch.float16, device=dev) for s in shapes5}
        big5 = max(shapes5, key=lambda s: binding.lib().mmd8_linear_workspace_bytes(M5, s.K, s.N))
        ws5 = binding.linear_workspace(M5, big5.K, big5.N, dev)
        last5 = shapes5[-1]
        ws5_exit = binding.linear_workspace(M5, last5.K, last5.N, dev, exit_block=block)
        codes_in5, absmax_in5 = binding.quantize_blockwise(X5[8192], block)       # the hidden state arrives encoded
        hidden5 = torch.empty((M5, 8192), dtype=torch.float16, device=dev)
        codes_out5 = torch.empty(M5 * last5.N, dtype=torch.uint8, device=dev)
        absmax_out5 = torch.empty((M5 * last5.N + block - 1) // block, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()

        def linear5(i, ev=None):
            shp = shapes5[i]
            if i == len(shapes5) - 1:
                # the last linear adds the residual stream (the decoded incoming hidden state) and encodes
                binding.mixed_int8_linear_to_codes(X5[shp.K], w5[i], wl.TAU, block, residual=hidden5, codes=codes_out5,
                                                   absmax=absmax_out5, workspace=ws5_exit, events=ev, tuning=tune)
            else:
                # the first linear takes the coded hidden state and decodes it
                binding.mixed_int8_linear(hidden5 if i == 0 else X5[shp.K], w5[i], wl.TAU, out=Y5[shp.name],
                                          workspace=ws5, events=ev, tuning=tune,
                                          coded=(codes_in5, absmax_in5, block) if i == 0 else None)

        def step5(events=None):
            for i in range(len(shapes5)):
                linear5(i, events[i] if events else None)

        ms_per_step = timed_wall(step5, args.steps, args.warmup, torch)
        ops5 = wl.linear_ops(M5, shapes5)
        tops = ops5 / (ms_per_step * 1e-3) / 1e12
        evs5 = [he.quad() for _ in shapes5]
        prep5, prep15, gemm5 = events_pass(step5, evs5, max(3, min(10, args.steps)), he, torch)
        gemm_tops5 = sum(2.0 * M5 * s.K * s.N for s in shapes5) / (sum(gemm5) * 1e-3) / 1e12
        per5 = {s.name: linear_row(M5, s, gemm5[i], prep5[i], prep15[i]) for i, s in enumerate(shapes5)}
        for i, s in enumerate(shapes5):
            # the whole call, back to back, no events recorded inside it (each record costs a few microseconds
            # between the kernels, which the prep_us / gemm_us split above includes)
            t_call = timed(lambda: linear5(i), 10)
            per5[s.name]["call_us"] = round(t_call * 1e3, 1)
            per5[s.name]["call_tops"] = round(2.0 * M5 * s.K * s.N / t_call / 1e9, 1)
            # what the preparation costs inside a call, where no event stands between the kernels
            per5[s.name]["call_minus_gemm_us"] = round(t_call * 1e3 - gemm5[i] * 1e3, 1)
        nel5 = M5 * 8192
        cb5 = 3.0 * nel5 + 4.0 * nel5 / block
        q5 = timed(lambda: binding.quantize_blockwise(Y5["o"], block, codes=codes_out5, absmax=absmax_out5))
        d5 = timed(lambda: binding.dequantize_blockwise(codes_in5, absmax_in5, block, out=hidden5.view(-1)))
        out.update({
            "metric": "mixed int8 linear TOPS (+% int8 MFMA peak); blockwise codec GB/s (+% HBM)",
            "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "int8", "data": "synthetic",
            "config": {"workload": "70B-shaped shard prefill (the largest single-GPU configuration): one decoder layer "
                                   "(QKV 8192->10240, O 8192->8192, gate/up 8192->57344, down 28672->8192), 4096 tokens, "
                                   "tau 6.0, 0.1%% outlier dims, W ~ N(0, 0.015^2); hidden state [4096,8192] decoded on "
                                   "entry and encoded on exit, block %d" % block,
                       "tokens": M5, "layers": 1, "codec_block": block},
            "pct_int8_peak": round(100.0 * tops / INT8_PEAK_TOPS, 2),
            "roofline": {"bound": "mfma", "kernel": "k_gemm_mixed (int8 MFMA GEMM + fused epilogue), the step's five launches (four linears; the 8192->10240 one takes two)",
                         "achieved": round(gemm_tops5, 2), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                         "frac": round(gemm_tops5 / INT8_PEAK_TOPS, 4), "traffic": gemm_traffic(),
                         "power_limited_ceiling": {"value": INT8_POWER_LIMITED_TOPS, "unit": "TOP/s",
                                                   "frac": round(gemm_tops5 / INT8_POWER_LIMITED_TOPS, 4),
                                                   "what": "register-only MFMA loop on Gaussian int8 codes under the "
                                                           "package power limit (no data movement); context next to "
                                                           "the nominal peak, which is what frac is quoted against"}},
            "per_linear": per5,
            "codec": {"step_tensor": {"quantize_gbs": round(cb5 / q5 / 1e6, 1), "dequantize_gbs": round(cb5 / d5 / 1e6, 1),
                                      "elements": nel5, "block": block,
                                      "note": "the step's own [4096,8192] hidden state, one buffer (served partly by the "
                                              "last-level cache)"}},
        })
        del w5, X5, Y5, ws5, ws5_exit, codes_in5, absmax_in5, hidden5, codes_out5, absmax_out5, X5h
        torch.cuda.empty_cache()

    # =================================================================== the 7B-shaped shard (2048 tokens): its weights
    # and inputs serve the second timed step and the decode, adapter, boundary and reading sections
    M = 2048
    shapes = wl.LLAMA_7B_LINEARS
    need_7b = any(want(n) for n in ("7b", "decode", "heavy", "readings", "adapter", "exit"))
    if need_7b:
        weights, Xs, Ys = [], {}, {}
        for layer in range(args.layers):
            row = []
            for i, shp in enumerate(shapes):
                W = torch.from_numpy(wl.prefill_weight(2, 20 + 10 * layer + i, shp, 0.02)).to(dev)
                row.append(binding.prequantize_weight(W))
                del W
            weights.append(row)
        for K in sorted({s.K for s in shapes}):
            X, _ = wl.prefill_activation(2, 10 + K % 5, M, K)
            Xs[K] = torch.from_numpy(X).to(dev)
        for shp in shapes:
            Ys[shp.name] = torch.empty((M, shp.N), dtype=torch.float16, device=dev)
        biggest = max(shapes, key=lambda s: binding.lib().mmd8_linear_workspace_bytes(M, s.K, s.N))
        workspace = binding.linear_workspace(M, biggest.K, biggest.N, dev)
        codes_in, absmax_in = binding.quantize_blockwise(Xs[4096], block)
        hidden_in = torch.empty((M, 4096), dtype=torch.float16, device=dev)
        codes_out = torch.empty(M * 4096, dtype=torch.uint8, device=dev)
        absmax_out = torch.empty((M * 4096 + block - 1) // block, dtype=torch.float32, device=dev)
        last = shapes[-1]                           # the shard's last linear hands its result on in coded form
        assert last.N == 4096
        ws_exit = binding.linear_workspace(M, last.K, last.N, dev, exit_block=block)
        torch.cuda.synchronize()

    if want("7b"):
        def step(events=None):
            n = 0
            for layer in range(args.layers):
                for i, shp in enumerate(shapes):
                    first = layer == 0 and i == 0
                    ev = events[n] if events else None
                    if layer == args.layers - 1 and i == len(shapes) - 1:
                        binding.mixed_int8_linear_to_codes(Xs[shp.K], weights[layer][i], wl.TAU, block, residual=hidden_in,
                                                           codes=codes_out, absmax=absmax_out, workspace=ws_exit, events=ev,
                                                           tuning=tune)
                    else:
                        binding.mixed_int8_linear(hidden_in if first else Xs[shp.K], weights[layer][i], wl.TAU,
                                                  out=Ys[shp.name], workspace=workspace, events=ev, tuning=tune,
                                                  coded=(codes_in, absmax_in, block) if first else None)
                    n += 1

        ms7 = timed_wall(step, args.steps, args.warmup, torch)
        ops7 = args.layers * wl.linear_ops(M, shapes)
        n_lin = args.layers * len(shapes)
        evs = [he.quad() for _ in range(n_lin)]
        prep_ms, prep1_ms, gemm_ms = events_pass(step, evs, max(3, min(10, args.steps)), he, torch)
        gemm_tops7 = sum(2.0 * M * s.K * s.N for _ in range(args.layers) for s in shapes) / (sum(gemm_ms) * 1e-3) / 1e12
        per7 = {}
        for j, shp in enumerate(shapes):
            mean = lambda v: float(np.mean([v[l * len(shapes) + j] for l in range(args.layers)]))
            per7[shp.name] = linear_row(M, shp, mean(gemm_ms), mean(prep_ms), mean(prep1_ms))
            # the whole (plain) call, back to back, the four layers' weights in turn, no events recorded inside it
            turn7 = [0]

            def call7():
                turn7[0] = (turn7[0] + 1) % args.layers
                binding.mixed_int8_linear(Xs[shp.K], weights[turn7[0]][j], wl.TAU, out=Ys[shp.name], workspace=workspace,
                                          tuning=tune)

            t_call = timed(call7, 12)
            per7[shp.name]["call_us"] = round(t_call * 1e3, 1)
            per7[shp.name]["call_tops"] = round(2.0 * M * shp.K * shp.N / t_call / 1e9, 1)
            per7[shp.name]["call_minus_gemm_us"] = round(t_call * 1e3 - mean(gemm_ms) * 1e3, 1)
        out["llama7b_prefill"] = {
            "workload": "Llama-7B-shaped shard prefill: %d decoder layers x (QKV 4096->12288, O 4096->4096, gate/up 4096->22016, "
                        "down 11008->4096), 2048 tokens, tau 6.0, 0.1%% outlier dims; hidden state [2048,4096] decoded on entry "
                        "and encoded on exit, block %d" % (args.layers, block),
            "ms_per_step": round(ms7, 4), "steps": args.steps, "value_tops": round(ops7 / (ms7 * 1e-3) / 1e12, 2),
            "pct_int8_peak": round(100.0 * ops7 / (ms7 * 1e-3) / 1e12 / INT8_PEAK_TOPS, 2),
            "gemm_tops": round(gemm_tops7, 2), "gemm_frac_of_int8_peak": round(gemm_tops7 / INT8_PEAK_TOPS, 4),
            "gemm_traffic_bytes_per_launch": gemm_traffic(GEMM_TRAFFIC_BYTES_PER_LAUNCH_7B), "per_linear": per7}
    dev_events = he.quad()
    genv = torch.Generator(device=dev)               # device-drawn tensors of the smaller sections
    genv.manual_seed(7)

    if want("codec"):
        # ---- the codec at the size of a shard-boundary hidden state [8192, 8192] (134 MB of fp16: HBM traffic, buffer
        # sets rotated so that nothing is served from the last-level cache); three tensors drawn by the host recipe
        nb, big = 3, 8192 * 8192
        xs_host = [torch.from_numpy(wl.boundary_hidden_state(tensor_id=t)[0]).view(-1) for t in range(nb)]
        xs = [h.to(dev) for h in xs_host]
        cs = [torch.empty(big, dtype=torch.uint8, device=dev) for _ in range(nb)]
        am = [torch.empty(big // 256, dtype=torch.float32, device=dev) for _ in range(nb)]
        turn, blk = [0], [block]

        def q_big():
            i = turn[0] = (turn[0] + 1) % nb
            binding.quantize_blockwise(xs[i], blk[0], codes=cs[i], absmax=am[i])

        def d_big():
            i = turn[0] = (turn[0] + 1) % nb
            binding.dequantize_blockwise(cs[i], am[i], blk[0], out=xs[i])

        def round_trip():
            q_big()
            binding.dequantize_blockwise(cs[turn[0]], am[turn[0]], blk[0], out=xs[turn[0]])

        by_block = {}
        for b in wl.CODEC_BLOCKS_BOUNDARY:
            blk[0] = b
            for i in range(nb):
                # every block size starts from the uploaded tensors: inputs that the decoder kernel wrote last are
                # encoded 10-15 % slower than uploaded ones whatever the block size (measured in any order of the sizes)
                xs[i].copy_(xs_host[i])
                binding.quantize_blockwise(xs[i], b, codes=cs[i], absmax=am[i])   # codes and scales of this block size
            # one buffer set over and over: served by the last-level cache as far as it fits (the "hot" figures);
            # both encoder timings come before the first decoder call of this block size
            tq = timed(q_big, 12)
            tq_hot = timed(lambda: binding.quantize_blockwise(xs[0], b, codes=cs[0], absmax=am[0]), 12)
            td = timed(d_big, 12)
            td_hot = timed(lambda: binding.dequantize_blockwise(cs[0], am[0], b, out=xs[0]), 12)
            trt = timed(round_trip, 12)
            nbytes = 3.0 * big + 4.0 * big / b
            by_block[str(b)] = {"quantize_gbs": round(nbytes / tq / 1e6, 1), "dequantize_gbs": round(nbytes / td / 1e6, 1),
                                "round_trip_gbs": round(2.0 * nbytes / trt / 1e6, 1),
                                "quantize_pct_hbm": round(100 * nbytes / tq / 1e6 / HBM_PEAK_GBS, 1),
                                "dequantize_pct_hbm": round(100 * nbytes / td / 1e6 / HBM_PEAK_GBS, 1),
                                "quantize_us": round(tq * 1e3, 1), "dequantize_us": round(td * 1e3, 1),
                                "hot_quantize_gbs": round(nbytes / tq_hot / 1e6, 1), "hot_dequantize_gbs": round(nbytes / td_hot / 1e6, 1)}
        # the other storage of the block scales (fp16 numbers, 2 bytes per block), smallest block: what it saves
        am16 = [torch.empty(big // 256, dtype=torch.float16, device=dev) for _ in range(nb)]

        def q_big16():
            i = turn[0] = (turn[0] + 1) % nb
            binding.quantize_blockwise(xs[i], 256, codes=cs[i], absmax=am16[i], fp16_scales=True)

        def d_big16():
            i = turn[0] = (turn[0] + 1) % nb
            binding.dequantize_blockwise(cs[i], am16[i], 256, out=xs[i])

        for i in range(nb):
            xs[i].copy_(xs_host[i])
            binding.quantize_blockwise(xs[i], 256, codes=cs[i], absmax=am16[i], fp16_scales=True)
        tq16, td16 = timed(q_big16, 12), timed(d_big16, 12)
        fp16_scales = {"block": 256, "quantize_us": round(tq16 * 1e3, 1), "dequantize_us": round(td16 * 1e3, 1),
                       "bytes_per_element": 3.0 + 2.0 / 256, "coded_fraction": (1 + 2.0 / 256) / 2,
                       "fp32_scales_quantize_us": by_block["256"]["quantize_us"],
                       "fp32_scales_dequantize_us": by_block["256"]["dequantize_us"]}
        del xs, xs_host, cs, am, am16
        out.setdefault("codec", {}).update({
            "fp16_block_scales": fp16_scales,
            "elements": big, "by_block": by_block,
            "note": "shard-boundary hidden state [8192,8192] (Student-t(3), 4 feature dimensions x50, host recipe), three buffer "
                    "sets taking turns (every call streams from HBM: the cold figures); hot_*: one buffer set over and over; "
                    "every block size starts from freshly uploaded tensors; the round trip runs last, on decoder-written values"})

    if want("decode"):
        # ---- decode shapes: the same linears with 1, 8, 32 and 64 tokens, heavy-tailed activations; the four layers' weights
        # take turns (360 MB of codes per shape family: cold)
        decode = {}
        decode_rows = (1, 8, 32, 64)
        for j, shp in enumerate(shapes):
            for Md in decode_rows:
                Xd = torch.from_numpy(wl.decode_activation(Md, Md, shp.K)).to(dev)
                Yd = torch.empty((Md, shp.N), dtype=torch.float16, device=dev)
                wsd = binding.linear_workspace(Md, shp.K, shp.N, dev)
                ts, ps = [], []
                for it in range(10):
                    binding.mixed_int8_linear(Xd, weights[it % args.layers][j], wl.TAU, out=Yd, workspace=wsd, events=dev_events)
                    torch.cuda.synchronize()
                    ps.append(he.elapsed_ms(dev_events[0], dev_events[1]))
                    ts.append(he.elapsed_ms(dev_events[1], dev_events[2]))
                t, pm = float(np.median(ts[2:])), float(np.median(ps[2:]))
                decode["%s_M%d" % (shp.name, Md)] = {"gemm_us": round(t * 1e3, 1), "prep_us": round(pm * 1e3, 1),
                                                      "weight_gbs": round(shp.K * shp.N / t / 1e6, 1),
                                                      "pct_hbm": round(100.0 * shp.K * shp.N / t / 1e6 / HBM_PEAK_GBS, 1),
                                                      "call_weight_gbs": round(shp.K * shp.N / (t + pm) / 1e6, 1)}

        # whole decoder layers, wall time of back-to-back calls (no events in between): all four layers' weights in turn,
        # 810 MB of codes per pass
        layer_bytes = float(sum(s.K * s.N for s in shapes))
        for Md in decode_rows:
            Xd = {K: torch.from_numpy(wl.decode_activation(Md, Md, K)).to(dev) for K in sorted({s.K for s in shapes})}
            Yd = {s.name: torch.empty((Md, s.N), dtype=torch.float16, device=dev) for s in shapes}
            big_d = max(shapes, key=lambda s: binding.lib().mmd8_linear_workspace_bytes(Md, s.K, s.N))
            wsd = binding.linear_workspace(Md, big_d.K, big_d.N, dev)

            def decode_pass():
                for layer in range(args.layers):
                    for j, shp in enumerate(shapes):
                        binding.mixed_int8_linear(Xd[shp.K], weights[layer][j], wl.TAU, out=Yd[shp.name], workspace=wsd)

            for _ in range(3):
                decode_pass()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(20):
                decode_pass()
            torch.cuda.synchronize()
            us = (time.perf_counter() - t0) / 20 / args.layers * 1e6
            decode["layer_M%d" % Md] = {"us_per_layer": round(us, 1), "weight_gbs": round(layer_bytes / us / 1e3, 1),
                                        "pct_hbm": round(100.0 * layer_bytes / us / 1e3 / HBM_PEAK_GBS, 1)}

    if want("heavy"):
        # ---- more than 128 rows of heavy-tailed input (hundreds of critical columns): the tiled GEMM's 16-bit part
        heavy = {}
        for Mh in (128, 256):                  # 128: the last size that still takes the decode kernels (two passes)
            Xh = {K: torch.from_numpy(wl.decode_activation(900 + Mh, Mh, K)).to(dev) for K in sorted({s.K for s in shapes})}
            Yh = {s.name: torch.empty((Mh, s.N), dtype=torch.float16, device=dev) for s in shapes}
            big_h = max(shapes, key=lambda s: binding.lib().mmd8_linear_workspace_bytes(Mh, s.K, s.N))
            wsh = binding.linear_workspace(Mh, big_h.K, big_h.N, dev)

            def heavy_pass():
                for j, shp in enumerate(shapes):
                    binding.mixed_int8_linear(Xh[shp.K], weights[0][j], wl.TAU, out=Yh[shp.name], workspace=wsh)

            heavy["layer_M%d_student_t" % Mh] = {"us_per_layer": round(timed(heavy_pass, 5) * 1e3, 1)}
        # the share of critical feature dimensions swept at 2048 tokens (Gaussian bulk, each critical dimension scaled by
        # U(8, 40)): critical columns travel as fp16 slabs of 32 through the GEMM's ring (the first 256 in slabs every
        # call has, up to 2048 more in further slabs), and from 2596 of these 4096 on (the last case) the GEMM kernel
        # makes a second, fp16 pass over K instead
        qkv = shapes[0]
        for share in (0.001, 0.008, 0.03, 0.06, 0.10, 0.25, 0.40, 0.70):
            Xm = torch.from_numpy(wl.gaussian_with_outlier_dims(M, qkv.K, share, 8.0, 40.0, wl.rng_for(2, 700))[0]).to(dev)
            t = timed(lambda: binding.mixed_int8_linear(Xm, weights[0][0], wl.TAU, out=Ys[qkv.name], workspace=workspace), 10)
            ps, gs = [], []
            for it in range(8):
                binding.mixed_int8_linear(Xm, weights[0][0], wl.TAU, out=Ys[qkv.name], workspace=workspace, events=dev_events)
                torch.cuda.synchronize()
                ps.append(he.elapsed_ms(dev_events[0], dev_events[1]))
                gs.append(he.elapsed_ms(dev_events[1], dev_events[2]))
            heavy["qkv_2048_tokens_%g_pct_critical" % (100 * share)] = {
                "critical_columns": int(round(share * qkv.K)), "call_us": round(t * 1e3, 1),
                "prep_us": round(float(np.median(ps[2:])) * 1e3, 1), "gemm_us": round(float(np.median(gs[2:])) * 1e3, 1),
                "call_tops": round(2.0 * M * qkv.K * qkv.N / (t * 1e-3) / 1e12, 1)}
            del Xm

    if want("readings"):
        # ---- the other readings of the layer (row scale over the non-critical columns only; original fp16 rows for the
        # critical dimensions): what each costs on the 7B-shaped QKV linear at 2048 tokens, whole calls
        qkv = shapes[0]
        W_master = torch.from_numpy(wl.prefill_weight(2, 20, qkv, 0.02)).to(dev)      # the matrix weights[0][0] was packed from
        readings = {}
        for name, rd in (("library", None), ("separate_scan_and_pack", (binding.ROW_SCALE_SUB_THRESHOLD, None)),
                         ("non_critical_row_scale", (binding.ROW_SCALE_NON_CRITICAL, None)),
                         ("fp16_master_rows", (binding.ROW_SCALE_SUB_THRESHOLD, W_master)),
                         ("both", (binding.ROW_SCALE_NON_CRITICAL, W_master))):
            t = timed(lambda: binding.mixed_int8_linear(Xs[qkv.K], weights[0][0], wl.TAU, out=Ys[qkv.name], workspace=workspace,
                                                        readings=rd), 20)
            readings[name] = {"call_us": round(t * 1e3, 1)}
        readings["note"] = ("QKV 4096->12288, 2048 tokens; the alternative readings run the scan and pack kernels separately "
                            "(5 bytes per element instead of 3), the non-critical scale one more pass over X; the master rows "
                            "cost 2 more resident bytes per weight, not time")
        del W_master

    if want("adapter"):
        # ---- the prefill linears with a rank-16 adapter (W' = W + B A, fp16 factors): "prep" now includes the
        # down-projection T = X A^T, the GEMM multiplies one more fp16 slab (T, B) per tile
        adapter, r_ad = {}, 16
        big_ad = max(shapes, key=lambda s: binding.lib().mmd8_linear_lora_workspace_bytes(M, s.K, s.N, r_ad))
        ws_ad = binding.linear_workspace(M, big_ad.K, big_ad.N, dev, lora_rank=r_ad)
        for j, shp in enumerate(shapes):
            A_np, B_np = wl.adapter_factors(2, 40 + j, shp.K, shp.N, r_ad)
            A_ad, B_ad = torch.from_numpy(A_np).to(dev), torch.from_numpy(B_np).to(dev)
            ts, ps = [], []
            for it in range(10):
                binding.mixed_int8_linear(Xs[shp.K], weights[it % args.layers][j], wl.TAU, out=Ys[shp.name], workspace=ws_ad,
                                          events=dev_events, lora=(A_ad, B_ad))
                torch.cuda.synchronize()
                ps.append(he.elapsed_ms(dev_events[0], dev_events[1]))
                ts.append(he.elapsed_ms(dev_events[1], dev_events[2]))
            t, pm = float(np.median(ts[2:])), float(np.median(ps[2:]))
            adapter[shp.name] = {"rank": r_ad, "gemm_us": round(t * 1e3, 1), "prep_us": round(pm * 1e3, 1),
                                 "gemm_tops": round(2.0 * M * shp.K * shp.N / t / 1e9, 1)}
        del ws_ad

    if want("exit"):
        # ---- the shard's last linear (down-projection + residual) handing on its result in coded form: one call
        # against layer, fp16 addition (a torch kernel) and encoder as three steps; whole calls, same buffers
        boundary_exit = {}
        for Mb in (M, 64, 1):
            Xb = Xs[last.K][:Mb] if Mb < M else Xs[last.K]
            Rb, Yb = hidden_in[:Mb], Ys[last.name][:Mb]
            Hb = torch.empty((Mb, last.N), dtype=torch.float16, device=dev)
            cb, ab = codes_out[:Mb * last.N], absmax_out
            wsb = binding.linear_workspace(Mb, last.K, last.N, dev, exit_block=block)

            def fused():
                binding.mixed_int8_linear_to_codes(Xb, weights[0][-1], wl.TAU, block, residual=Rb, codes=cb, absmax=ab,
                                                   workspace=wsb)

            def separate():
                binding.mixed_int8_linear(Xb, weights[0][-1], wl.TAU, out=Yb, workspace=wsb)
                torch.add(Yb, Rb, out=Hb)
                binding.quantize_blockwise(Hb, block, codes=cb, absmax=ab)

            def with_residual():                  # the same linear inside the shard: residual added, fp16 out
                binding.mixed_int8_linear(Xb, weights[0][-1], wl.TAU, out=Hb, workspace=wsb, residual=Rb)

            def layer_then_add():
                binding.mixed_int8_linear(Xb, weights[0][-1], wl.TAU, out=Yb, workspace=wsb)
                torch.add(Yb, Rb, out=Hb)

            boundary_exit["M%d" % Mb] = {"one_call_us": round(timed(fused, 30) * 1e3, 1),
                                         "three_steps_us": round(timed(separate, 30) * 1e3, 1), "block": block,
                                         "residual_one_call_us": round(timed(with_residual, 30) * 1e3, 1),
                                         "residual_two_steps_us": round(timed(layer_then_add, 30) * 1e3, 1)}

    if want("vit"):
        # ---- ViT-L-shaped block (width 1024, 8 images x 197 tokens, bias everywhere): the four linears, the first
        # MLP linear with GELU applied in its own kernels against the same layer followed by a separate fp16
        # activation kernel (torch's).  Weights N(0, 0.02^2) drawn on the device, whole calls.
        vit, Mv = {}, 8 * 197
        for shp in wl.VIT_L_LINEARS:
            Wv = torch.empty((shp.K, shp.N), dtype=torch.float16, device=dev).normal_(0.0, 0.02, generator=genv)
            pwv = binding.prequantize_weight(Wv)
            del Wv
            Xv = torch.empty((Mv, shp.K), dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=genv)
            Xv[:, :2] *= 20.0
            bv = torch.empty(shp.N, dtype=torch.float16, device=dev).normal_(0.0, 0.1, generator=genv)
            Yv = torch.empty((Mv, shp.N), dtype=torch.float16, device=dev)
            wsv = binding.linear_workspace(Mv, shp.K, shp.N, dev)
            t = timed(lambda: binding.mixed_int8_linear(Xv, pwv, wl.TAU, bias=bv, out=Yv, workspace=wsv), 30)
            vit[shp.name] = {"call_us": round(t * 1e3, 1), "tops": round(2.0 * Mv * shp.K * shp.N / t / 1e9, 1)}
            if shp.name == "fc1":
                def two_steps():
                    binding.mixed_int8_linear(Xv, pwv, wl.TAU, bias=bv, out=Yv, workspace=wsv)
                    torch.nn.functional.gelu(Yv)

                vit["fc1_gelu"] = {
                    "one_call_us": round(timed(lambda: binding.mixed_int8_linear(Xv, pwv, wl.TAU, bias=bv, out=Yv,
                                                                                 workspace=wsv, gelu=True), 30) * 1e3, 1),
                    "two_steps_us": round(timed(two_steps, 30) * 1e3, 1)}
        vit["tokens"] = Mv

    if want("prequant"):
        # ---- weight pre-quantization (offline step, not part of the timed step): column absmax + codes in the blocked
        # layout; 2 bytes read twice and 1 byte written per weight
        prequant = {}
        for shp in shapes:
            Wp = torch.empty((shp.K, shp.N), dtype=torch.float16, device=dev).normal_(0.0, 0.02, generator=genv)
            t = timed(lambda: binding.prequantize_weight(Wp), 5)
            prequant[shp.name] = {"us": round(t * 1e3, 1), "gbs": round(5.0 * shp.K * shp.N / t / 1e6, 1),
                                  "pct_hbm": round(100.0 * 5.0 * shp.K * shp.N / t / 1e6 / HBM_PEAK_GBS, 1)}
            del Wp

    if want("kv"):
        # ---- the codec on a key/value cache (one layer of the 7B shape: 32 heads x 128, block = one head vector):
        # a 2048-token context decoded for one generated token (K and V), one token appended, a 2048-token prompt
        # appended.  Whole calls, eager; the cache of this one layer fits the last-level cache.
        Hh, Dh, Tc = 32, 128, 2048
        kv_x = [torch.empty((Tc, Hh, Dh), dtype=torch.float16, device=dev).normal_(0.0, 1.0, generator=genv) for _ in range(2)]
        kv_c = [torch.empty((Tc, Hh, Dh), dtype=torch.uint8, device=dev) for _ in range(2)]
        kv_a = [torch.empty((Tc, Hh), dtype=torch.float32, device=dev) for _ in range(2)]

        def kv_append(t0, n):                      # views made once: the timed calls are the library's alone
            views = [(kv_x[i][t0:t0 + n], kv_c[i][t0:t0 + n].view(-1), kv_a[i][t0:t0 + n].view(-1)) for i in range(2)]

            def run():
                for x, c, a in views:
                    binding.quantize_blockwise(x, Dh, codes=c, absmax=a)
            return run

        kv_read_views = [(kv_c[i].view(-1), kv_a[i].view(-1), kv_x[i].view(-1)) for i in range(2)]

        def kv_read():
            for c, a, x in kv_read_views:
                binding.dequantize_blockwise(c, a, Dh, out=x)

        kv_append(0, Tc)()
        kv_bytes = 2.0 * (3.0 + 4.0 / Dh) * Tc * Hh * Dh
        t_read, t_tok, t_prompt = timed(kv_read, 30), timed(kv_append(Tc - 1, 1), 30), timed(kv_append(0, Tc), 30)
        kv_cache = {"heads": Hh, "head_dim": Dh, "context": Tc,
                    "read_context_us": round(t_read * 1e3, 1), "read_context_gbs": round(kv_bytes / t_read / 1e6, 1),
                    "append_token_us": round(t_tok * 1e3, 1),
                    "append_prompt_us": round(t_prompt * 1e3, 1), "append_prompt_gbs": round(kv_bytes / t_prompt / 1e6, 1),
                    "coded_fraction": (1 + 4.0 / Dh) / 2,
                    "note": "two calls (K and V) each; at these sizes a call is bound by its launch and the Python "
                            "binding (about 7 us of host time per call), not by the kernel (3-6 us)"}
        del kv_x, kv_c, kv_a, kv_read_views

    for key, name in (("decode", "decode"), ("heavy_tailed_prefill", "heavy"), ("readings", "readings"), ("adapter", "adapter"),
                      ("boundary_exit", "boundary_exit"), ("vit_l_block", "vit"), ("kv_cache", "kv_cache"),
                      ("weight_prequant", "prequant")):
        if name in locals():
            out[key] = locals()[name]
    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)            # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    if need_7b:
        del weights, Xs, Ys
    torch.cuda.empty_cache()
    if not args.no_cpu_baseline and want("step"):
        out["cpu_baseline"] = cpu_baseline(cpu_sample, hidden_host, block)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
