"""The Muon step can be captured into a HIP graph: a captured step replayed k times leaves exactly the weights and
momentum that k eager steps leave.  Replays are separated by unrelated eager work and synchronisations, and every
replay is checked (a graph that is only right on its first replay would pass a single comparison)."""
from __future__ import annotations

import pytest
import torch

from paper_2502_16982_amd import binding, workloads
from tests.gpu_util import hp_from

pytestmark = pytest.mark.gpu

CASES = {
    "bf16_mixed": dict(shapes=[(128, 256), (384, 256), (200, 136), (256, 640)], ns_dtype="bf16",
                       w_dtype=torch.bfloat16, g_dtype=torch.bfloat16),
    # two bf16 planes; the 256 x 256 instantiations of this path use per-lane scratch memory in their epilogue
    "bf16x2_mixed": dict(shapes=[(512, 640), (384, 256), (200, 136)], ns_dtype="bf16x2",
                         w_dtype=torch.bfloat16, g_dtype=torch.bfloat16),
    "f32_single": dict(shapes=[(128, 256)], ns_dtype="f32", w_dtype=torch.float32, g_dtype=torch.float32),
}


@pytest.mark.parametrize("case", sorted(CASES))
def test_captured_step_replays_like_eager_steps(case):
    dev = torch.device("cuda:0")
    cfg = CASES[case]
    wl = workloads.custom(case, cfg["shapes"], w_dtype=cfg["w_dtype"], g_dtype=cfg["g_dtype"], ns_dtype=cfg["ns_dtype"],
                          seed_base=4200)
    tensors = workloads.make_all(wl, dev)
    hp, _ = hp_from(wl.hyper)
    st = binding.MuonStepper(tensors, ns_dtype=wl.ns_dtype)
    rms = torch.zeros(len(tensors), dtype=torch.float32, device=dev)
    side = torch.cuda.Stream(device=dev)
    try:
        side.wait_stream(torch.cuda.current_stream(dev))
        with torch.cuda.stream(side):
            st.step(hp, stream=side, update_rms=rms)          # warm-up: uploads the pointer table
        side.synchronize()
        w0 = [t[0].clone() for t in tensors]
        m0 = [t[2].clone() for t in tensors]

        eager = []
        for _ in range(3):
            with torch.cuda.stream(side):
                st.step(hp, stream=side, update_rms=rms)
            side.synchronize()
            eager.append(([t[0].clone() for t in tensors], [t[2].clone() for t in tensors], rms.clone()))

        for t, w, m in zip(tensors, w0, m0):
            t[0].copy_(w)
            t[2].copy_(m)
        torch.cuda.synchronize(dev)

        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            st.step(hp, stream=side, update_rms=rms)
        # capturing enqueues nothing: the state is still the snapshot
        torch.cuda.synchronize(dev)
        for t, w in zip(tensors, w0):
            assert torch.equal(t[0], w)

        scratch = torch.zeros(1 << 16, device=dev)
        for k in range(3):
            graph.replay()
            torch.cuda.synchronize(dev)
            scratch.add_(1.0)                                  # unrelated eager work between replays
            assert float(scratch.sum().item()) == (k + 1) * scratch.numel()
            torch.cuda.synchronize(dev)
            ew, em, erms = eager[k]
            for i, t in enumerate(tensors):
                assert torch.equal(t[0], ew[i]), f"{case}: W of matrix {i} differs after replay {k + 1}"
                assert torch.equal(t[2], em[i]), f"{case}: M of matrix {i} differs after replay {k + 1}"
            assert torch.equal(rms, erms), f"{case}: update RMS differs after replay {k + 1}"
    finally:
        st.close()
