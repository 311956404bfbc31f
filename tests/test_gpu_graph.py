"""The library's calls allocate nothing and synchronise nothing, so a sequence of them can be captured in a
HIP graph (a decode step is launch-bound: four short kernels per linear).  A graph of four decode-shaped
linears, a prefill-shaped linear, a codec round trip and two linears whose result leaves in coded form is replayed several times, with eager work and
synchronisation between the replays and with new input values written into the captured buffers; every
replay must equal the eager result bit for bit."""
import numpy as np
import pytest
import torch

from paper_2407_19775_amd import binding, workloads as wl
from gpu_util import to_gpu

pytestmark = pytest.mark.gpu


def test_graph_replays_equal_eager_calls():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(0)
    shapes = [(1, 512, 1024), (8, 1024, 520), (64, 528, 264), (40, 2048, 512), (300, 1040, 520)]
    block = 256
    pws, Xs, wss, Ys = [], [], [], []
    for (M, K, N) in shapes:
        pws.append(binding.prequantize_weight(to_gpu(wl.gaussian_weight(K, N, 0.02, rng))))
        Xs.append(torch.empty((M, K), dtype=torch.float16, device=dev))
        wss.append(binding.linear_workspace(M, K, N, dev))
        Ys.append(torch.empty((M, N), dtype=torch.float16, device=dev))
    n_last = Ys[-1].numel()
    codes = torch.empty(n_last, dtype=torch.uint8, device=dev)
    absmax = torch.empty((n_last + block - 1) // block, dtype=torch.float32, device=dev)
    back = torch.empty(n_last, dtype=torch.float16, device=dev)
    # coded exits: a decode-shaped one (shape 3, residual) and a tiled one
    Xe = torch.empty((300, 528), dtype=torch.float16, device=dev)
    pwe = binding.prequantize_weight(to_gpu(wl.gaussian_weight(528, 512, 0.02, rng)))
    exits = []
    for (X, pw, blk) in [(Xs[3], pws[3], 256), (Xe, pwe, 128)]:
        M, N = X.shape[0], pw.N
        exits.append(dict(X=X, pw=pw, block=blk, R=torch.empty((M, N), dtype=torch.float16, device=dev),
                          codes=torch.empty(M * N, dtype=torch.uint8, device=dev),
                          absmax=torch.empty(M * N // blk, dtype=torch.float32, device=dev),
                          ws=binding.linear_workspace(M, X.shape[1], N, dev, exit_block=blk)))

    def fill_inputs(seed):
        r = np.random.default_rng(seed)
        for X in Xs + [Xe] + [e["R"] for e in exits]:
            x = r.standard_t(3.0, size=tuple(X.shape)).astype(np.float32)
            X.copy_(to_gpu(wl.to_fp16(x)))

    def run():
        for X, pw, ws, Y in zip(Xs, pws, wss, Ys):
            binding.mixed_int8_linear(X, pw, wl.TAU, out=Y, workspace=ws)
        binding.quantize_blockwise(Ys[-1], block, codes=codes, absmax=absmax)
        binding.dequantize_blockwise(codes, absmax, block, out=back)
        for e in exits:
            binding.mixed_int8_linear_to_codes(e["X"], e["pw"], wl.TAU, e["block"], residual=e["R"], codes=e["codes"],
                                               absmax=e["absmax"], workspace=e["ws"])

    outputs = Ys + [codes, absmax, back] + [e["codes"] for e in exits] + [e["absmax"] for e in exits]

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in outputs]

    fill_inputs(1)
    torch.cuda.synchronize()                # no warm-up call: setting up the workspaces prepared the kernels
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for seed in (1, 2, 3, 4):
        fill_inputs(seed)
        run()
        eager = snapshot()
        for t in outputs:
            t.fill_(0)                      # the replay must produce everything again
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        for i, (a, b) in enumerate(zip(eager, replayed)):
            assert torch.equal(a.view(torch.uint8) if a.dtype != torch.uint8 else a,
                               b.view(torch.uint8) if b.dtype != torch.uint8 else b), ("output", i, "seed", seed)
        # eager work of the program's own between the replays
        binding.mixed_int8_linear(Xs[1], pws[1], wl.TAU, out=Ys[1], workspace=wss[1])
        torch.cuda.synchronize()
