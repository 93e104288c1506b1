"""The library's calls under HIP graph capture: nothing on the hot path allocates, synchronises or clears
memory with a memset node, so an encode + decode (two-pass kernels and the single-read coder) and a whole
iteration can be captured once and replayed.  Every replay is held against the eager call bit for bit,
with eager work of the same context and synchronisations between the replays."""
import pytest
import torch

from gpu_util import DEV, buffers, say
from paper_1901_08227_amd import binding as B
from paper_1901_08227_amd import synth

pytestmark = pytest.mark.gpu


def _same(a, b):
    return all(torch.equal(a[k], b[k]) for k in ("codes", "scales", "vbar"))


@pytest.mark.parametrize("M,d,bits,norm", [(8, 4096 * 37 + 20, 4, B.NORM_QUOT),   # two-pass kernels, ragged rows
                                           (8, 1 << 23, 2, B.NORM_SUB)])          # the coder that reads g once
def test_encode_decode_replayed_from_a_graph(M, d, bits, norm):
    g, gref = synth.codec_inputs(M, d, 5, device=DEV)
    torch.cuda.synchronize()
    side = torch.cuda.Stream(device=DEV)
    ctx = B.Context(d=d, M=M, bits=bits, norm=norm, seed=3, device=DEV, stream=side)
    eager, other, replayed = buffers(ctx), buffers(ctx), buffers(ctx)
    torch.cuda.synchronize()  # the buffers were filled on the current stream, the context works on its own
    it = 6
    with torch.cuda.stream(side):
        ctx.normalize_encode(it, g, gref, eager["codes"], eager["scales"])
        ctx.decode_aggregate(eager["codes"], eager["scales"], gref, eager["vbar"])
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.normalize_encode(it, g, gref, replayed["codes"], replayed["scales"])
            ctx.decode_aggregate(replayed["codes"], replayed["scales"], gref, replayed["vbar"])
        for k in range(3):
            say(f"graph replay {k}: d={d} M={M} bits={bits} norm={norm}")
            for t in replayed.values():
                t.zero_()
            # eager work of the same context in between: another iteration number into other buffers
            ctx.normalize_encode(it + 1 + k, g, gref, other["codes"], other["scales"])
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert _same(eager, replayed), f"replay {k} differs from the eager call"
            assert not torch.equal(other["codes"], eager["codes"])
    ctx.close()


def test_whole_iteration_replayed_from_a_graph():
    # Rosenbrock chain with the noise generated on the device: nothing but the library's own kernels
    M, d = 8, 1 << 18
    side = torch.cuda.Stream(device=DEV)
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, seed=1, lr=1e-5, ref_policy=B.REF_LAST_AVG, ref_period=1,
                    problem=B.PROB_ROSENBROCK, device=DEV, stream=side)
    ctx.set_noise_variance(0.01)
    w0 = synth.rosenbrock_start(d, 1, device=DEV)
    r0 = torch.randn(d, generator=torch.Generator(device=DEV).manual_seed(2), device=DEV) * 0.1
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        eager, replayed = buffers(ctx), buffers(ctx)
        w_e, r_e, w_r, r_r = w0.clone(), r0.clone(), w0.clone(), r0.clone()
        torch.cuda.synchronize()
        ctx.step(4, w_e, r_e, eager["g"], eager["codes"], eager["scales"], eager["vbar"])
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            ctx.step(4, w_r, r_r, replayed["g"], replayed["codes"], replayed["scales"], replayed["vbar"])
        for k in range(3):
            say(f"graph replay {k} of a whole iteration")
            w_r.copy_(w0)
            r_r.copy_(r0)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert _same(eager, replayed) and torch.equal(eager["g"], replayed["g"]), f"replay {k}"
            assert torch.equal(w_e, w_r) and torch.equal(r_e, r_r), f"replay {k}: iterate or reference"
    ctx.close()
