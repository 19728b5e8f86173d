"""GPU parity of muon_adamw_step (through the C ABI) against the fp64 AdamW oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import adamw_oracle as ao  # noqa: E402
from paper_2502_16982_amd import binding  # noqa: E402
from tests import gpu_util as U  # noqa: E402


@pytest.fixture(scope="module")
def dev():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    binding.lib()
    return torch.device("cuda:0")


def make(sizes, p_dtype, g_dtype, dev, seed):
    gen = torch.Generator(device=dev)
    gen.manual_seed(seed)
    out = []
    for n in sizes:
        p = torch.empty(n, device=dev).normal_(0, 0.5, generator=gen).to(p_dtype)
        g = torch.empty(n, device=dev).normal_(0, 1e-2, generator=gen).to(g_dtype)
        out.append((p, g, torch.zeros(n, device=dev), torch.zeros(n, device=dev)))
    return out


@pytest.mark.parametrize("p_dtype,g_dtype", [(torch.float32, torch.float32), (torch.bfloat16, torch.bfloat16),
                                             (torch.float32, torch.bfloat16)])
def test_adamw_parity_multi_tensor_three_steps(dev, p_dtype, g_dtype):
    # ragged sizes: below one vector, one span, several spans with a tail, and more than 24 tensors (two launches)
    sizes = [1, 3, 4096, 4097, 10000, 123457] + [257 + 31 * i for i in range(24)]
    tensors = make(sizes, p_dtype, g_dtype, dev, 100)
    host = [[U.to64(t) for t in quad] for quad in tensors]
    hp = dict(lr=3e-3, weight_decay=0.1, beta1=0.9, beta2=0.95, eps=1e-8)
    for step in (1, 2, 3):
        if step > 1:
            gen = torch.Generator(device=dev)
            gen.manual_seed(1000 + step)
            for k, quad in enumerate(tensors):
                quad[1].copy_(torch.empty(quad[1].numel(), device=dev).normal_(0, 1e-2, generator=gen).to(g_dtype))
                host[k][1] = U.to64(quad[1])
        binding.muon_adamw_step(tensors, step=step, stream_ptr=torch.cuda.current_stream(dev).cuda_stream, **hp)
        torch.cuda.synchronize()
        for k, quad in enumerate(tensors):
            p0, g0, m0, v0 = host[k]
            pr, mr, vr = ao.adamw_step(p0, g0, m0, v0, step=step, **hp)
            m_gpu, v_gpu = U.to64(quad[2]), U.to64(quad[3])
            assert np.max(np.abs(m_gpu - mr) / (np.abs(0.9 * m0) + np.abs(0.1 * g0) + 1e-300)) <= U.TOL_ELEM
            assert np.max(np.abs(v_gpu - vr) / (np.abs(0.95 * v0) + np.abs(0.05 * g0 * g0) + 1e-300)) <= U.TOL_ELEM
            # parameter: feed the library's own moments to the oracle's last line, as for Muon's weight update
            bc1, bc2 = 1 - 0.9 ** step, 1 - 0.95 ** step
            upd = (m_gpu / bc1) / (np.sqrt(v_gpu / bc2) + hp["eps"])
            ref = p0 - hp["lr"] * (upd + hp["weight_decay"] * p0)
            got = U.to64(quad[0])
            scale = np.abs(p0) + hp["lr"] * np.abs(upd)
            if p_dtype == torch.float32:
                assert np.max(np.abs(got - ref) / scale) <= 2 * U.TOL_ELEM
            else:
                diff = np.abs(got - U.bf16_round(ref))
                assert (diff / U.bf16_ulp(ref)).max() <= 1.0 and np.mean(diff > 0) <= 5e-3
            host[k] = [got, g0, m_gpu, v_gpu]


def test_adamw_degenerate_and_errors(dev):
    L = binding.lib()
    p = torch.randn(5000, device=dev)
    p0 = p.clone()
    z = torch.zeros_like(p)
    m, v = z.clone(), z.clone()
    binding.muon_adamw_step([(p, z, m, v)], lr=0.5, weight_decay=0.1, step=1)     # zero gradient: pure decay, no NaN
    torch.cuda.synchronize()
    assert torch.isfinite(p).all() and torch.count_nonzero(m).item() == 0 and torch.count_nonzero(v).item() == 0
    assert torch.allclose(p, p0 * 0.95, rtol=1e-6, atol=0)
    q = p.clone()
    binding.muon_adamw_step([(p, torch.randn_like(p), m, v)], lr=0.0, weight_decay=0.1, step=2)   # lr = 0
    torch.cuda.synchronize()
    assert torch.equal(p, q) and torch.count_nonzero(m).item() > 0
    arr = (binding.muon_adamw_param * 1)()
    arr[0].p, arr[0].g, arr[0].m, arr[0].v = p.data_ptr(), z.data_ptr(), m.data_ptr(), v.data_ptr()
    arr[0].numel, arr[0].p_dtype, arr[0].g_dtype = 5000, 0, 0
    ok = binding.muon_adamw_hparams(0.1, 0.1, 0.9, 0.95, 1e-8, 1)
    assert L.muon_adamw_step(arr, 1, C.byref(ok), None) == 0
    assert L.muon_adamw_step(None, 1, C.byref(ok), None) == -1
    assert L.muon_adamw_step(arr, 0, C.byref(ok), None) == -1
    assert L.muon_adamw_step(arr, 1, C.byref(binding.muon_adamw_hparams(0.1, 0.1, 0.9, 0.95, 1e-8, 0)), None) == -1
    assert L.muon_adamw_step(arr, 1, C.byref(binding.muon_adamw_hparams(0.1, 0.1, 1.0, 0.95, 1e-8, 1)), None) == -1
    arr[0].p_dtype = 7
    assert L.muon_adamw_step(arr, 1, C.byref(ok), None) == -2
    arr[0].p_dtype = 0
    arr[0].m = m.data_ptr() + 2
    assert L.muon_adamw_step(arr, 1, C.byref(ok), None) == -7
    arr[0].m = m.data_ptr()
    arr[0].numel = 0
    assert L.muon_adamw_step(arr, 1, C.byref(ok), None) == -1
    torch.cuda.synchronize()
