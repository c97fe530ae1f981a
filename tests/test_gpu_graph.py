"""The layer step under HIP graph capture: the header promises that every entry point only enqueues
kernels on the caller's stream (no allocation, no synchronization, no second stream), so a forward +
backward pass recorded once must replay correctly.  Each replay runs on new input contents, with eager
work and a synchronization between the replays, and is compared bit for bit with the same calls made
eagerly on separate buffers (those are what the parity tests check against the oracle)."""
import pytest
import torch

from paper_2501_17116_amd import binding as b
from paper_2501_17116_amd import synth

pytestmark = pytest.mark.gpu


def _inputs(seed, M, K, N, dtype):
    g = torch.Generator().manual_seed(seed)
    A = torch.randn(M, K, generator=g)
    A[:, (7 * seed + 3) % K] *= 40.0
    dY = torch.randn(M, N, generator=g) * 0.01
    cast = torch.bfloat16 if dtype == "bf16" else torch.float32
    return synth._finish(A, dtype).to(cast).cuda(), synth._finish(dY, dtype).to(cast).cuda()


@pytest.mark.parametrize("scope", [b.FP4_OCC_TENSOR, b.FP4_OCC_TOKEN])
@pytest.mark.parametrize("dtype,cached", [("bf16", False), ("bf16", True), ("f32", False)])
def test_layer_step_replays_from_a_graph(dtype, cached, scope):
    M, K, N, alpha = 640, 1024, 544, 0.99
    cast = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(99)
    W = synth._finish(torch.randn(K, N, generator=g) * 0.02, dtype).to(cast).cuda()
    sets = [_inputs(s, M, K, N, dtype) for s in (1, 2, 3)]

    # static buffers of the recorded step
    A, dY = torch.empty_like(sets[0][0]), torch.empty_like(sets[0][1])
    Y = torch.empty((M, N), dtype=cast, device="cuda")
    dA = torch.empty((M, K), dtype=cast, device="cuda")
    dW = torch.empty((K, N), dtype=torch.float32, device="cuda")
    ctx = b.FwdCtx(M, K, N, alpha, scope=scope)
    ws = b.Workspace()
    ws.get(max(b.workspace_bytes(op, M, K, N, b._dt(A)) for op in (b.FP4_OP_FWD, b.FP4_OP_BWD, b.FP4_OP_PREPARE)))
    wq = b.fp4_prepare_weights(W, ws=ws) if cached else None

    def step():
        if cached:
            b.fp4_linear_fwd_cached(A, W, wq, alpha, ctx=ctx, Y=Y, ws=ws)
        else:
            b.fp4_linear_fwd(A, W, alpha, ctx=ctx, Y=Y, ws=ws)
        b.fp4_linear_bwd(dY, A, W, ctx, 5.0, 3.0, wq=wq, dA=dA, dW=dW, ws=ws)

    A.copy_(sets[0][0])
    dY.copy_(sets[0][1])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                  # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()

    for rep, (A_s, dY_s) in enumerate(sets + sets[:1]):
        A.copy_(A_s)                            # eager work between the replays
        dY.copy_(dY_s)
        Y.zero_(); dA.zero_(); dW.zero_()
        graph.replay()
        torch.cuda.synchronize()
        # the same calls, eagerly, on buffers of their own
        ctx2 = b.FwdCtx(M, K, N, alpha, scope=scope)
        Y2, _ = b.fp4_linear_fwd(A_s, W, alpha, ctx=ctx2)
        dA2, dW2 = b.fp4_linear_bwd(dY_s, A_s, W, ctx2, 5.0, 3.0)
        torch.cuda.synchronize()
        nnz = int(ctx2.nnz.item())
        assert int(ctx.nnz.item()) == nnz > 0, rep
        assert torch.equal(ctx.row_ptr, ctx2.row_ptr), rep
        assert torch.equal(ctx.col_idx[:nnz], ctx2.col_idx[:nnz]) and torch.equal(ctx.val[:nnz], ctx2.val[:nnz]), rep
        assert torch.equal(ctx.thresholds, ctx2.thresholds), rep
        assert torch.equal(Y, Y2), rep
        assert torch.equal(dA, dA2), rep
        assert torch.equal(dW, dW2), rep
