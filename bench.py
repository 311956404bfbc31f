"""Benchmark of the compressed-shard hot path on one MI355X.

A step is one pass of a Llama-7B-shaped shard over one prefill batch: the incoming hidden state
is decoded from its blockwise 8-bit form (inside the first linear's preparation kernel), the 16
linears of 4 decoder layers (QKV 4096->12288,
O 4096->4096, gate/up 4096->22016, down 11008->4096; 2048 tokens) run through the mixed int8
decomposition (scan, pack, int8 GEMM with fused epilogue), and the outgoing hidden state (the last
linear's output plus the residual stream) is encoded again in that linear's epilogue.  Weights are pre-quantized before the timed region (they are static).  Inputs are
seeded synthetic tensors resident in HBM.  Prints one JSON line.
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
# HBM bytes per GEMM launch (mean over the five launches of a decoder layer) from rocprofv3 FETCH_SIZE and
# WRITE_SIZE, scaled by a plain copy of known size (profiles/gemm_llama7b_prefill_hbm_traffic.txt).  Valid
# for the GEMM source it was measured on: reported as null once that file has changed.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = 200.0e6
GEMM_TRAFFIC_SOURCE_SHA256 = "99b6dffbde06008ff7fea89490783a3113f389fdbbe2116e245f541079ff32a1"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--codec-block", type=int, default=256)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-step", action="store_true",
                    help="profiling aid: skip the extra sections (large codec tensor, decode, 70B, adapter)")
    ap.add_argument("--gemm-variant", type=int, default=-1, help="tuning: force a GEMM tile configuration (-1 = automatic)")
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

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        assert self.hip.hipEventElapsedTime(ctypes.byref(ms), a, b) == 0
        return ms.value


def gemm_traffic():
    import hashlib
    src = os.path.join(ROOT, "paper_2407_19775_amd", "csrc", "gemm_kernels.hip")
    try:
        same = hashlib.sha256(open(src, "rb").read()).hexdigest() == GEMM_TRAFFIC_SOURCE_SHA256
    except OSError:
        same = False
    return GEMM_TRAFFIC_BYTES_PER_LAUNCH if same else None


def cpu_baseline(wl, passes=4):
    """The CPU oracle on a bounded sample of the same workload: the step's sixteen linears at full size
    (one decoder layer's tensors, `passes` times: the oracle's time does not depend on the values) plus as
    many codec round trips of one hidden state."""
    import numpy as np
    from oracle import blockwise_codec as bc
    from oracle import mixed_linear as ml
    ops = 0
    M = 2048
    prepared = []
    for i, shp in enumerate(wl.LLAMA_7B_LINEARS):
        X, _ = wl.prefill_activation(2, 10 + shp.K % 5, M, shp.K)
        W = wl.prefill_weight(2, 20 + i, shp, 0.02)
        Wq, c = ml.prequantize_weight(W)             # offline step, untimed like on the GPU
        prepared.append((X, Wq, c))
        ops += 2 * M * shp.K * shp.N
    hidden = prepared[0][0]
    t0 = time.perf_counter()
    for _ in range(passes):
        codes, a = bc.quantize_blockwise(hidden, 1024)
        bc.dequantize_blockwise(codes, a, 1024)
        for X, Wq, c in prepared:
            ml.mixed_int8_linear(X, Wq, c, wl.TAU)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count()
    return {"value": passes * ops / dt / 1e12, "unit": "TOPS", "cores": int(cores), "kind": "oracle",
            "sample": "%d passes over one decoder layer (4 linears, 2048 tokens, full size) + as many codec round "
                      "trips of one [2048,4096] hidden state: the step's amount of work; %.1f s" % (passes, dt)}


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
    M = 2048
    shapes = wl.LLAMA_7B_LINEARS
    block = args.codec_block

    # ---- static state: pre-quantized weights (distinct per layer), inputs, outputs, workspaces
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
    # incoming hidden state arrives encoded
    codes_in, absmax_in = binding.quantize_blockwise(Xs[4096], block)
    hidden_in = torch.empty((M, 4096), dtype=torch.float16, device=dev)
    codes_out = torch.empty(M * 4096, dtype=torch.uint8, device=dev)
    absmax_out = torch.empty((M * 4096 + block - 1) // block, dtype=torch.float32, device=dev)
    last = shapes[-1]                           # the shard's last linear hands its result on in coded form
    assert last.N == 4096
    ws_exit = binding.linear_workspace(M, last.K, last.N, dev, exit_block=block)
    torch.cuda.synchronize()

    def step(events=None):
        n = 0
        for layer in range(args.layers):
            for i, shp in enumerate(shapes):
                first = layer == 0 and i == 0      # the shard's first linear takes the coded hidden state and decodes it
                if layer == args.layers - 1 and i == len(shapes) - 1:
                    # the last one adds the residual stream (here: the decoded incoming hidden state) and encodes
                    binding.mixed_int8_linear_to_codes(Xs[shp.K], weights[layer][i], wl.TAU, block, residual=hidden_in,
                                                       codes=codes_out, absmax=absmax_out, workspace=ws_exit,
                                                       events=events[n] if events else None)
                else:
                    binding.mixed_int8_linear(hidden_in if first else Xs[shp.K], weights[layer][i], wl.TAU,
                                              out=Ys[shp.name], workspace=workspace, events=events[n] if events else None,
                                              coded=(codes_in, absmax_in, block) if first else None)
                n += 1

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    ops_per_step = args.layers * wl.linear_ops(M, shapes)
    tops = ops_per_step / (ms_per_step * 1e-3) / 1e12

    # ---- second pass with events around every GEMM kernel (roofline of the dominant kernel) and
    # around the codec kernels
    he = HipEvents()
    n_lin = args.layers * len(shapes)
    evs = [[he.create() for _ in range(3)] for _ in range(n_lin)]
    gemm_ms, prep_ms = [0.0] * n_lin, [0.0] * n_lin
    reps = max(3, min(10, args.steps))
    for _ in range(reps):
        step(evs)
        torch.cuda.synchronize()
        for i, (e0, e1, e2) in enumerate(evs):
            prep_ms[i] += he.elapsed_ms(e0, e1) / reps
            gemm_ms[i] += he.elapsed_ms(e1, e2) / reps
    gemm_ops = [2.0 * M * s.K * s.N for _ in range(args.layers) for s in shapes]
    gemm_tops = sum(gemm_ops) / (sum(gemm_ms) * 1e-3) / 1e12
    per_shape = {}
    for j, shp in enumerate(shapes):
        ms = np.mean([gemm_ms[l * len(shapes) + j] for l in range(args.layers)])
        pm = np.mean([prep_ms[l * len(shapes) + j] for l in range(args.layers)])
        per_shape[shp.name] = {"gemm_us": round(ms * 1e3, 1), "gemm_tops": round(2.0 * M * shp.K * shp.N / ms / 1e9, 1),
                               "prep_us": round(pm * 1e3, 1),
                               "prep_gbs": round(3.0 * M * shp.K / pm / 1e6, 1)}

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

    nel = M * 4096
    codec_bytes = 3.0 * nel + 4.0 * nel / block
    q_ms = timed(lambda: binding.quantize_blockwise(Ys["down"], block, codes=codes_out, absmax=absmax_out))
    d_ms = timed(lambda: binding.dequantize_blockwise(codes_in, absmax_in, block, out=hidden_in.view(-1)))

    if not args.only_step:
        # ---- the codec at the size of a shard-boundary hidden state [8192, 8192] (134 MB of fp16: HBM
        # traffic, buffers rotated so that nothing is served from the last-level cache)
        nb, big = 3, 8192 * 8192
        gen4 = torch.Generator(device=dev)
        gen4.manual_seed(4)

        def student_t3(n):
            # Student-t with 3 degrees of freedom drawn on the device: z / sqrt(chi2_3 / 3)
            z = torch.randn(n, device=dev, generator=gen4)
            c2 = torch.zeros(n, device=dev)
            for _ in range(3):
                c2 += torch.randn(n, device=dev, generator=gen4) ** 2
            return z * torch.rsqrt(c2 / 3.0)

        xs = []
        for _ in range(nb):
            t = student_t3(big).view(8192, 8192)
            t[:, torch.randint(0, 8192, (4,), device=dev, generator=gen4)] *= 50.0     # 0.05 % of the feature dimensions
            xs.append(t.clamp_(-65504.0, 65504.0).to(torch.float16).view(-1))
            del t
        cs = [torch.empty(big, dtype=torch.uint8, device=dev) for _ in range(nb)]
        am = [torch.empty(big // 256, dtype=torch.float32, device=dev) for _ in range(nb)]
        big_bytes = 3.0 * big + 4.0 * big / block
        turn = [0]
        blk = [block]

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
        for b in (256, 1024, 4096):
            blk[0] = b
            for i in range(nb):                                   # codes and scales of this block size in every buffer
                binding.quantize_blockwise(xs[i], b, codes=cs[i], absmax=am[i])
            tq, td, trt = timed(q_big, 12), timed(d_big, 12), timed(round_trip, 12)
            nbytes = 3.0 * big + 4.0 * big / b
            by_block[str(b)] = {"quantize_gbs": round(nbytes / tq / 1e6, 1), "dequantize_gbs": round(nbytes / td / 1e6, 1),
                                "round_trip_gbs": round(2.0 * nbytes / trt / 1e6, 1),
                                "quantize_pct_hbm": round(100 * nbytes / tq / 1e6 / HBM_PEAK_GBS, 1),
                                "dequantize_pct_hbm": round(100 * nbytes / td / 1e6 / HBM_PEAK_GBS, 1)}
        blk[0] = block
        for i in range(nb):
            binding.quantize_blockwise(xs[i], block, codes=cs[i], absmax=am[i])
        qb_ms, db_ms = timed(q_big, 12), timed(d_big, 12)
        del xs, cs, am

        # ---- decode shapes: the same linears with 1 and 64 tokens, heavy-tailed activations; the four
        # layers' weights take turns (360 MB of codes per shape family: cold)
        decode = {}
        dev_events = [he.create() for _ in range(3)]
        for j, shp in enumerate(shapes):
            for Md in (1, 64):
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
                                                      "pct_hbm": round(100.0 * shp.K * shp.N / t / 1e6 / HBM_PEAK_GBS, 1)}

        # whole decoder layers at 1 and 64 tokens, wall time of back-to-back calls (no events in between):
        # all four layers' weights in turn, 810 MB of codes per pass
        layer_bytes = float(sum(s.K * s.N for s in shapes))
        for Md in (1, 8, 64):
            Xd = {K: torch.from_numpy(wl.decode_activation(Md, Md, K)).to(dev) for K in sorted({s.K for s in shapes})}
            Yd = {s.name: torch.empty((Md, s.N), dtype=torch.float16, device=dev) for s in shapes}
            wsd = binding.linear_workspace(Md, biggest.K, biggest.N, dev)

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

        # ---- ViT-L-shaped block (width 1024, 8 images x 197 tokens, bias everywhere): the four linears, the first
        # MLP linear with GELU applied in its own kernels against the same layer followed by a separate fp16
        # activation kernel (torch's).  Weights N(0, 0.02^2) drawn on the device, whole calls.
        vit, Mv = {}, 8 * 197
        genv = torch.Generator(device=dev)
        genv.manual_seed(7)
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

        # ---- weight pre-quantization (offline step, not part of the timed step): column absmax + codes in the blocked
        # layout; 2 bytes read twice and 1 byte written per weight
        prequant = {}
        for shp in shapes:
            Wp = torch.empty((shp.K, shp.N), dtype=torch.float16, device=dev).normal_(0.0, 0.02, generator=genv)
            t = timed(lambda: binding.prequantize_weight(Wp), 5)
            prequant[shp.name] = {"us": round(t * 1e3, 1), "gbs": round(5.0 * shp.K * shp.N / t / 1e6, 1),
                                  "pct_hbm": round(100.0 * 5.0 * shp.K * shp.N / t / 1e6 / HBM_PEAK_GBS, 1)}
            del Wp

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

        # ---- 70B-shaped shard prefill (4096 tokens, one decoder layer: 856 MB of weight codes), per linear:
        # preparation and GEMM time from the library's events.  Weights drawn on the device (N(0, 0.015^2)).
        del weights, Xs, Ys
        torch.cuda.empty_cache()
        prefill_70b, M5 = {}, 4096
        gen = torch.Generator(device=dev)
        gen.manual_seed(5)
        ops5 = t5 = 0.0
        for shp in wl.LLAMA_70B_LINEARS:
            W = torch.empty((shp.K, shp.N), dtype=torch.float16, device=dev)
            W.normal_(0.0, 0.015, generator=gen)
            pw5 = binding.prequantize_weight(W)
            del W
            X5, _ = wl.prefill_activation(5, 10 + shp.K % 5, M5, shp.K)
            X5 = torch.from_numpy(X5).to(dev)
            Y5 = torch.empty((M5, shp.N), dtype=torch.float16, device=dev)
            ws5 = binding.linear_workspace(M5, shp.K, shp.N, dev)
            ts, ps = [], []
            for it in range(7):
                binding.mixed_int8_linear(X5, pw5, wl.TAU, out=Y5, workspace=ws5, events=dev_events)
                torch.cuda.synchronize()
                ps.append(he.elapsed_ms(dev_events[0], dev_events[1]))
                ts.append(he.elapsed_ms(dev_events[1], dev_events[2]))
            t, pm = float(np.median(ts[2:])), float(np.median(ps[2:]))
            o5 = 2.0 * M5 * shp.K * shp.N
            ops5, t5 = ops5 + o5, t5 + t + pm
            prefill_70b[shp.name] = {"gemm_us": round(t * 1e3, 1), "gemm_tops": round(o5 / t / 1e9, 1),
                                     "pct_int8_peak": round(100.0 * o5 / t / 1e9 / INT8_PEAK_TOPS, 1),
                                     "prep_us": round(pm * 1e3, 1), "prep_gbs": round(3.0 * M5 * shp.K / pm / 1e6, 1)}
            del pw5, X5, Y5, ws5
        prefill_70b["layer_tops_end_to_end"] = round(ops5 / t5 / 1e9, 1)

    out = {
        "metric": "mixed int8 linear TOPS (+% int8 MFMA peak); blockwise codec GB/s (+% HBM)",
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "Llama-7B-shaped shard prefill: %d decoder layers x (QKV 4096->12288, O 4096->4096, "
                               "gate/up 4096->22016, down 11008->4096), 2048 tokens, tau 6.0, 0.1%% outlier dims; "
                               "hidden state [2048,4096] decoded on entry and encoded on exit, block %d"
                               % (args.layers, block),
                   "tokens": M, "layers": args.layers, "codec_block": block},
        "pct_int8_peak": round(100.0 * tops / INT8_PEAK_TOPS, 2),
        "roofline": {"bound": "mfma", "kernel": "k_gemm_mixed (int8 MFMA GEMM + fused epilogue)",
                     "achieved": round(gemm_tops, 2), "peak": INT8_PEAK_TOPS, "unit": "TOP/s",
                     "frac": round(gemm_tops / INT8_PEAK_TOPS, 4), "traffic": gemm_traffic()},
        "per_linear": per_shape,
        "codec": {"step_tensor": {"quantize_gbs": round(codec_bytes / q_ms / 1e6, 1),
                                  "dequantize_gbs": round(codec_bytes / d_ms / 1e6, 1), "elements": nel, "block": block,
                                  "note": "the step's own [2048,4096] hidden state: 25 MB per call, launch-bound"}},
    }
    if not args.only_step:
        out["codec"].update({
            "quantize_gbs": round(big_bytes / qb_ms / 1e6, 1), "dequantize_gbs": round(big_bytes / db_ms / 1e6, 1),
            "quantize_pct_hbm": round(100 * big_bytes / qb_ms / 1e6 / HBM_PEAK_GBS, 1),
            "dequantize_pct_hbm": round(100 * big_bytes / db_ms / 1e6 / HBM_PEAK_GBS, 1),
            "elements": big, "block": block,
            "by_block": by_block,
            "note": "shard-boundary hidden state [8192,8192] (Student-t(3), 4 feature dimensions x50), three buffer "
                    "sets taking turns (HBM traffic); after the first pass the values are codec outputs"})
        out.update({"decode": decode, "prefill_70b": prefill_70b, "adapter": adapter, "boundary_exit": boundary_exit,
                    "vit_l_block": vit, "kv_cache": kv_cache, "weight_prequant": prequant})
    if args.calibrate_copy:
        src = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)            # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
