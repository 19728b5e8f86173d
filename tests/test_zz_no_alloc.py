"""muon_step_static, the entry point that allocates nothing (its workspace is a fixed device array inside the
library), against muon_init + muon_step on the same inputs: bitwise-equal W, M and update RMS, on two calls in a row,
the second with a smaller input (another shape list, so the scratch is re-planned and holds the first call's leftovers),
then two more steps of the first list (plan switched back, momentum carried)."""
import ctypes as C

import pytest
import torch

pytestmark = pytest.mark.gpu

from paper_2502_16982_amd import binding, workloads  # noqa: E402


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    return torch.device("cuda:0")


def params_of(tensors):
    arr = (binding.muon_param * len(tensors))()
    for i, (w, g, m) in enumerate(tensors):
        arr[i].w, arr[i].g, arr[i].m = w.data_ptr(), g.data_ptr(), m.data_ptr()
        arr[i].rows, arr[i].cols = w.shape
        arr[i].w_dtype, arr[i].g_dtype = binding.dtype_code(w.dtype), binding.dtype_code(g.dtype)
    return arr


def run_pair(wl, dev, ns, steps, hp):
    """`steps` steps through muon_step_static and through muon_init/muon_step on clones; returns both states."""
    a = workloads.make_all(wl, dev)
    b = [tuple(t.clone() for t in trip) for trip in a]
    n = len(a)
    rms_a = torch.zeros(n, device=dev)
    rms_b = torch.zeros(n, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    pa = params_of(a)
    st = binding.MuonStepper(b, ns_dtype=ns)
    for s in range(steps):
        if s:
            for i in range(n):
                g = workloads.make_gradient(wl, i, s, dev)
                a[i][1].copy_(g)
                b[i][1].copy_(g)
        binding.muon_step_static(pa, n, binding.NS_DTYPES[ns], hp, stream, rms_a.data_ptr())
        st.step(hp, update_rms=rms_b)
    torch.cuda.synchronize()
    st.close()
    return a, b, rms_a, rms_b


def assert_same(a, b, rms_a, rms_b):
    for (wa, _, ma), (wb, _, mb) in zip(a, b):
        assert torch.equal(wa, wb) and torch.equal(ma, mb)
    assert torch.equal(rms_a, rms_b)
    assert torch.isfinite(rms_a).all() and (rms_a > 0).all()


@pytest.mark.parametrize("ns", ["bf16", "bf16x2", "f32"])
def test_static_matches_workspace_entry_point(dev, ns):
    hp = binding.default_hparams(lr=0.02, weight_decay=0.1)
    big = workloads.custom("static_big_" + ns, [(512, 768), (768, 512), (640, 1408), (200, 333)], ns_dtype=ns, seed_base=91)
    small = workloads.custom("static_small_" + ns, [(256, 384), (100, 60)], ns_dtype=ns, seed_base=92)
    assert_same(*run_pair(big, dev, ns, 2, hp))
    assert_same(*run_pair(small, dev, ns, 1, hp))      # smaller input right after: other plan, leftovers in the scratch
    assert_same(*run_pair(big, dev, ns, 2, hp))


def test_static_limits_and_errors(dev):
    L = binding.lib()
    hp = binding.default_hparams(lr=0.02)
    # more workspace than the array holds: rejected before anything is enqueued, buffers untouched
    w = torch.ones(4096, 4096, dtype=torch.bfloat16, device=dev)
    g = torch.ones_like(w)
    m = torch.zeros(4096, 4096, device=dev)
    p = params_of([(w, g, m)])
    assert L.muon_step_static(p, 1, binding.MUON_BF16, C.byref(hp), None, None) == -9
    torch.cuda.synchronize()
    assert torch.count_nonzero(m).item() == 0 and torch.equal(w, torch.ones_like(w))
    # more matrices than the pointer pack holds
    tiny = [(torch.zeros(8, 8, device=dev), torch.ones(8, 8, device=dev), torch.zeros(8, 8, device=dev)) for _ in range(65)]
    assert L.muon_step_static(params_of(tiny), 65, binding.MUON_F32, C.byref(hp), None, None) == -9
    assert L.muon_step_static(params_of(tiny), 64, binding.MUON_F32, C.byref(hp), None, None) == 0
    torch.cuda.synchronize()
    # argument errors
    assert L.muon_step_static(None, 1, binding.MUON_BF16, C.byref(hp), None, None) == -1
    assert L.muon_step_static(params_of(tiny), 1, 7, C.byref(hp), None, None) == -2
    assert L.muon_step_static(params_of(tiny), 1, binding.MUON_F32, None, None, None) == -1
    nul = params_of(tiny[:1])
    nul[0].w = None
    assert L.muon_step_static(nul, 1, binding.MUON_F32, C.byref(hp), None, None) == -1
    assert L.muon_status_string(-9).decode() != "unknown status"
