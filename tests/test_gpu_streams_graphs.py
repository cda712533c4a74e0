"""The calls are asynchronous on the caller's stream and, in flat mode, consist of kernel launches only:
they run on a side stream next to other work, and they can be recorded into a HIP graph and replayed."""
import numpy as np
import pytest
import torch

from oracle import oracle
from paper_2305_12201_amd import binding, workloads
from tests.gpu_util import STAT_RTOL

pytestmark = pytest.mark.gpu


def _same_bits(a, b):
    return np.array_equal(np.asarray(a).view(np.uint32), np.asarray(b).view(np.uint32))


def test_side_stream_next_to_work_on_the_default_stream():
    n, cfs, commit = 1_500_007, [50.0, 500.0], 0
    grad = workloads.resnet_like_gradient(n, seed=41)
    res0 = workloads.normal_gradient(n, 1e-5, seed=42)
    comp = binding.Compressor(n, cfs, commit)
    g = torch.from_numpy(grad).cuda()
    r = torch.from_numpy(res0.copy()).cuda()
    dense = torch.zeros(n, dtype=torch.float32, device="cuda")
    dws = torch.empty(binding.gravac_decompress_workspace_bytes(1, n), dtype=torch.uint8, device="cuda")
    busy = torch.ones(8_000_000, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    side = torch.cuda.Stream()                      # default priority
    for _ in range(20):                             # unrelated work queued on the default stream
        busy.mul_(1.0001)
    with torch.cuda.stream(side):
        idx, val, stats = comp(g, r)                # stream=None -> the current (side) stream
        binding.gravac_decompress_accumulate(idx, val, [idx.numel()], dense, workspace=dws, stream=side)
    side.synchronize()
    assert binding.gravac_read_status(comp.workspace, stream=side)["internal_error"] == 0
    ref_res = res0.copy()
    ref_idx, ref_val, ref_stats = oracle.compress(grad, ref_res, cfs, commit)
    ref_dense = np.zeros(n, np.float32)
    oracle.decompress_accumulate(ref_idx, ref_val, [ref_idx.size], ref_dense)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert _same_bits(val.cpu().numpy(), ref_val)
    assert _same_bits(r.cpu().numpy(), ref_res)
    assert _same_bits(dense.cpu().numpy(), ref_dense)
    np.testing.assert_allclose(stats.cpu().numpy()[..., :3], ref_stats[..., :3], rtol=STAT_RTOL, atol=0)
    torch.cuda.synchronize()


def test_flat_compress_and_decompress_replayed_from_a_graph():
    """One iteration (compress, then decompress of the fresh message) is captured once and replayed for five
    iterations with new gradients, the residual carried on the device; the program's own eager work and
    synchronisations sit between the replays; every replay is checked against the oracle."""
    n, cfs, commit = 1_200_011, [100.0, 1000.0], 0
    comp = binding.Compressor(n, cfs, commit)
    k = comp.k_total
    g = torch.zeros(n, dtype=torch.float32, device="cuda")          # static input buffer of the graph
    r = torch.zeros(n, dtype=torch.float32, device="cuda")          # residual, carried from replay to replay
    dense = torch.zeros(n, dtype=torch.float32, device="cuda")
    dws = torch.empty(binding.gravac_decompress_workspace_bytes(1, n), dtype=torch.uint8, device="cuda")
    grads = [workloads.resnet_like_gradient(n, seed=60 + i) for i in range(6)]

    # one eager iteration first (what a program does before it captures)
    g.copy_(torch.from_numpy(grads[0]))
    comp(g, r)
    binding.gravac_decompress_accumulate(comp.out_idx, comp.out_val, [k], dense, workspace=dws)
    torch.cuda.synchronize()
    ref_res = np.zeros(n, np.float32)
    ref_dense = np.zeros(n, np.float32)
    ri, rv, _ = oracle.compress(grads[0], ref_res, cfs, commit)
    oracle.decompress_accumulate(ri, rv, [ri.size], ref_dense)
    assert _same_bits(r.cpu().numpy(), ref_res)

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        comp(g, r)                                                   # launches go to the capturing stream
        binding.gravac_decompress_accumulate(comp.out_idx, comp.out_val, [k], dense, workspace=dws)
    # capturing executes nothing: residual and dense buffer are still those of the eager iteration
    torch.cuda.synchronize()
    assert _same_bits(r.cpu().numpy(), ref_res)

    for it in range(1, 6):
        g.copy_(torch.from_numpy(grads[it]))                         # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ri, rv, rs = oracle.compress(grads[it], ref_res, cfs, commit)
        oracle.decompress_accumulate(ri, rv, [ri.size], ref_dense)
        assert np.array_equal(comp.out_idx.cpu().numpy(), ri), f"replay {it}: indices"
        assert _same_bits(comp.out_val.cpu().numpy(), rv), f"replay {it}: values"
        assert _same_bits(r.cpu().numpy(), ref_res), f"replay {it}: residual"
        assert _same_bits(dense.cpu().numpy(), ref_dense), f"replay {it}: dense buffer"
        np.testing.assert_allclose(comp.out_stats.cpu().numpy()[..., :3], rs[..., :3], rtol=STAT_RTOL, atol=0)
        assert int(comp.out_count.item()) == k
        assert comp.status()["internal_error"] == 0


def test_calls_that_cannot_be_replayed_refuse_a_capturing_stream():
    n = 300_000
    seg = np.array([0, 100_000, 100_064, n], dtype=np.int64)
    comp_seg = binding.Compressor(n, [100.0], 0, seg)
    comp_flat = binding.Compressor(n, [100.0], 0)
    g = torch.from_numpy(workloads.normal_gradient(n, 1e-3, seed=5)).cuda()
    r = torch.zeros(n, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    timer = binding.CallTimer()
    graph = torch.cuda.CUDAGraph()
    codes = []
    with torch.cuda.graph(graph):
        for comp, tm in ((comp_seg, None), (comp_flat, timer)):
            try:
                comp(g, r, timer=tm)
                codes.append(0)
            except binding.GravacError as e:
                codes.append(e.code)
        comp_flat(g, r)                                              # so that the graph is not empty
    assert codes == [binding.ERR_CAPTURE, binding.ERR_CAPTURE]
    torch.cuda.synchronize()
