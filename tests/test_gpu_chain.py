"""GPU parity of agq_gemm_chain_* (a chain of quantized linear layers in one launch) against the CPU oracle.

Every stage is checked on the tensor that really flowed into it: the oracle's layer (Eq.2, integer product,
per-channel dequantization) is applied to the caller's input or to the fp16 output the GPU wrote for the stage
before; accumulators must match bit for bit, fp16 outputs to the tolerance of the other GEMM tests."""
from __future__ import annotations

import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

from paper_2312_05693_amd import synth  # noqa: E402
from test_gpu_parity import assert_f16_close, dev, host  # noqa: E402


@pytest.fixture(scope="module")
def agq():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2312_05693_amd import binding
    binding.lib()
    return binding


def build_chain(agq, oracle, M, spec, seed, scale_unit=True):
    """spec: list of (K, [N...], src) with src = None (a caller tensor) or the projection of the stage before.
    Exponents come from an oracle pass over the chain (calibration), weights from the input recipe with scales
    divided so that activations keep unit size along the chain.  Returns (stages for the binding, host copies)."""
    stages, hosts = [], []
    prev_y = None
    for s, (K, Ns, src) in enumerate(spec):
        if src is None:
            x = synth.make_activation(M, K, 2, seed=seed + 31 * s)
        else:
            x = prev_y[src]
        bits = 4 if (s % 5 == 3) else 8
        e = oracle.calibrate_act_exp(x, bits)
        projs_h, projs_d, ys = [], [], []
        for p, N in enumerate(Ns):
            wq, sw = synth.make_weight_q4(N, K, seed=seed + 7 * s + p)
            if scale_unit:
                sw = (sw.astype(np.float32) / (0.02 * np.sqrt(K))).astype(np.float16)
            projs_h.append((wq, sw))
            acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
            projs_d.append((agq.pack_w4(dev(wq)), dev(sw), N, None, acc))
            ys.append(oracle.linear_w4(x, bits, e, 0, wq, sw)[1])
        stages.append(dict(x=dev(x) if src is None else None, src_proj=src or 0, bits=bits, e=e, K=K, projs=projs_d))
        hosts.append(dict(x=x if src is None else None, src=src, bits=bits, e=e, K=K, projs=projs_h))
        prev_y = ys
    return stages, hosts


def check_chain(agq, oracle, M, stages, hosts, plan):
    assert agq.gemm_chain_status(plan) == agq.AGQ_OK
    prev = None
    for s, (st, h) in enumerate(zip(stages, hosts)):
        x_in = h["x"] if h["src"] is None else prev[h["src"]]
        outs = []
        for p, (wq, sw) in enumerate(h["projs"]):
            acc_w, y_w = oracle.linear_w4(x_in, h["bits"], h["e"], 0, wq, sw)
            acc_g = host(st["projs"][p][4])
            y_g = host(plan.ys[s][p])
            assert np.array_equal(acc_g.astype(np.int64), acc_w), "stage %d projection %d: accumulators" % (s, p)
            assert_f16_close(y_g, y_w, "stage %d projection %d" % (s, p))
            outs.append(y_g)
        prev = outs


@pytest.mark.parametrize("M", [1, 2, 3, 4])
def test_chain_small(agq, oracle, M):
    # external input, three projections; then chains through different projections, a 4-bit stage (s = 3), a second
    # caller tensor in the middle, a ragged K split (1408 = 11 chunks over 8 wavefronts), one chunk only (128)
    spec = [(256, [384, 128, 256], None), (128, [512], 1), (512, [256, 1408], 0), (1408, [128, 48], 1),
            (128, [640], 0), (768, [256], None), (256, [16], 0)]
    stages, hosts = build_chain(agq, oracle, M, spec, seed=300 + M)
    plan = agq.gemm_chain_prepare(stages, M)
    agq.gemm_chain_run(plan)
    check_chain(agq, oracle, M, stages, hosts, plan)


def test_chain_many_tiles_and_long_k(agq, oracle):
    # more than eight tiles per workgroup (two rounds), the longest K, and the LLaMA-7B down projection's K
    M = 3
    spec = [(128, [40000, 16384], None), (16384, [11008], 1), (11008, [256, 128], 0)]
    stages, hosts = build_chain(agq, oracle, M, spec, seed=411)
    plan = agq.gemm_chain_prepare(stages, M)
    agq.gemm_chain_run(plan)
    check_chain(agq, oracle, M, stages, hosts, plan)


def test_chain_replays_with_new_inputs_and_graph(agq, oracle):
    """The same prepared workspace, run again after the caller's input tensor changed (eagerly, then from a captured
    graph): every run starts a new range of epochs, so no record of an earlier run can be taken for a new one."""
    M = 4
    spec = [(512, [256, 256], None), (256, [384], 1), (384, [512], 0), (512, [128], 0)]
    stages, hosts = build_chain(agq, oracle, M, spec, seed=520)
    plan = agq.gemm_chain_prepare(stages, M)
    x_dev = stages[0]["x"]
    graph = None
    for rep in range(6):
        if rep > 0:
            x_new = synth.make_activation(M, 512, 2, seed=9000 + rep)
            hosts[0]["x"] = x_new
            x_dev.copy_(dev(x_new))
        for st in stages:                       # outputs of the previous run must not survive by accident
            for pr in st["projs"]:
                pr[4].zero_()
        for outs in plan.ys:
            for y in outs:
                y.zero_()
        torch.cuda.synchronize()
        if rep < 3:
            agq.gemm_chain_run(plan)
        else:
            if graph is None:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    agq.gemm_chain_run(plan)
            graph.replay()
        check_chain(agq, oracle, M, stages, hosts, plan)


@pytest.mark.parametrize("M", [1, 4])
def test_chain_llama7b_two_blocks(agq, oracle, M):
    """Two LLaMA-7B blocks as one chain, the benchmark's wiring: q/k/v from the block input, o on the output of q
    (the attention output has that shape), gate/up on the output of o, down on the output of gate, and the next
    block's q/k/v on the output of down."""
    d, F = 4096, 11008
    spec = []
    for blk in range(2):
        spec += [(d, [d, d, d], None if blk == 0 else 0), (d, [d], 0), (d, [F, F], 0), (F, [d], 0)]
    stages, hosts = build_chain(agq, oracle, M, spec, seed=77 + M)
    plan = agq.gemm_chain_prepare(stages, M)
    agq.gemm_chain_run(plan)
    check_chain(agq, oracle, M, stages, hosts, plan)
