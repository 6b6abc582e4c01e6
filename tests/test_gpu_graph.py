"""Library calls under HIP graph capture: a captured forward + backward of a decomposed linear layer
(split-K weight gradients, padded raw rank, GELU epilogues) and of a Tucker convolution must replay to
the same bits as eager launches, on every replay, with eager work and synchronisation in between
(the library clears nothing with memset and allocates nothing, so a capture holds kernels only)."""
import pytest
import torch

import synth_inputs as si
from parity import dev, empty, f32, workspace
from paper_2309_03824_amd import binding as lrd

pytestmark = pytest.mark.gpu


def _replay_matches_eager(step, outputs):
    """step(): launches on the current stream; outputs: tensors it writes."""
    step()
    torch.cuda.synchronize()
    want = [t.clone() for t in outputs]
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    torch.cuda.synchronize()
    for rep in range(4):
        for t in outputs:
            t.fill_(float(rep + 1))            # eager work between the replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outputs, want):
            assert torch.equal(got, ref), rep
        step()                                  # an eager step between replays
        torch.cuda.synchronize()
        for got, ref in zip(outputs, want):
            assert torch.equal(got, ref), rep


@pytest.mark.parametrize("r", [192, 61])
def test_linear_pair_replays_bit_exact(r):
    dt, T, n_in, n_out = "bf16", 2048, 768, 3072
    rng = si.rng_for(2, 700 + r)
    X, dY = dev(si.gaussian((T, n_in), rng), dt), dev(si.gaussian((T, n_out), rng), dt)
    U, V = si.direct_factors(n_out, n_in, r, rng)
    U, V = dev(U, dt), dev(V, dt)
    bias = torch.from_numpy(si.gaussian((n_out,), rng).astype("float32")).cuda()
    Y, A, H, dX = empty((T, n_out), dt), empty((T, n_out), dt), empty((T, r), dt), empty((T, n_in), dt)
    dV, dU, db = f32((r, n_in)), f32((n_out, r)), f32((n_out,))
    ws = workspace(lrd.linear_workspace_bytes(T, n_in, n_out, r, lrd.BF16, 0))

    def step():
        lrd.linear_fwd_act(X, V, U, bias, Y, A, H, lrd.ACT_GELU, ws)
        lrd.linear_bwd_act(dY, X, H, V, U, dX, dV, dU, db, 0, X, lrd.ACT_GELU, ws)

    _replay_matches_eager(step, [Y, A, H, dX, dV, dU, db])


def test_tucker_conv_replays_bit_exact():
    dt = "bf16"
    N, hw, C, S, r1, r2, k = 4, 14, 64, 96, 32, 40, 3
    g = lrd.conv_geom(N, hw, hw, C, S, r1, r2, k, 1, 1)
    rng = si.rng_for(4, 701)
    X, dY = dev(si.gaussian((N, hw, hw, C), rng), dt), dev(si.gaussian((N, hw, hw, S), rng), dt)
    P1, G, P2 = si.direct_tucker_factors(S, C, k, r1, r2, rng)
    P1, G, P2 = dev(P1, dt), dev(G, dt), dev(P2, dt)
    Y, A, B, dX = empty((N, hw, hw, S), dt), empty((N, hw, hw, r1), dt), empty((N, hw, hw, r2), dt), empty((N, hw, hw, C), dt)
    dP1, dG, dP2 = f32((r1, C)), f32((r2, k, k, r1)), f32((S, r2))
    ws = workspace(lrd.tucker_conv_workspace_bytes(g, lrd.BF16, 0))

    def step():
        lrd.tucker_conv_fwd(X, P1, G, P2, Y, A, B, g, ws)
        lrd.tucker_conv_bwd(dY, X, A, B, P1, G, P2, dX, dP1, dG, dP2, 0, g, ws)

    _replay_matches_eager(step, [Y, A, B, dX, dP1, dG, dP2])
