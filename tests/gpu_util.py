"""Helpers for the GPU parity tests: run the HIP library through its C ABI and the fp64 oracle on the
very same seeded buffers, and measure the errors the tolerances are stated in."""
from __future__ import annotations

import numpy as np
import torch

from oracle import muon_oracle as orc
from paper_2502_16982_amd import binding, workloads

TOL_F32_FRO = 1e-4      # relative Frobenius error of O, fp32 Newton-Schulz path
TOL_BF16_FRO = 2e-2     # relative Frobenius error of O, bf16 Newton-Schulz path
# split-bf16 paths: the fp32 path's bar for two planes (each product is good to about 2^-16), a tighter one for three
# planes (what is left is the fp32 accumulation and the fp32 epilogue arithmetic)
TOL_SPLIT_FRO = {"bf16x2": 1e-4, "bf16x3": 1e-5}
TOL_ELEM = 1e-6         # elementwise momentum / update error relative to the sum of term magnitudes


def to64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def hp_from(h: workloads.Hyper, **over):
    d = dict(lr=h.lr, weight_decay=h.weight_decay, momentum=h.momentum, a=h.a, b=h.b, c=h.c,
             rms_scale=h.rms_scale, eps=h.eps, ns_steps=h.ns_steps, nesterov=int(h.nesterov),
             scale_mode=binding.MUON_SCALE_ADJUSTED_LR, hidden_size=0.0)
    d.update(over)
    if d.get("coeff_schedule") is not None:
        d["ns_steps"] = len(d["coeff_schedule"])
    return binding.default_hparams(**d), d


SCALE_MODE_NAMES = {0: "adjusted_lr", 1: "baseline", 2: "update_norm"}


def oracle_step(w0, g0, m0, d):
    return orc.muon_step(w0, g0, m0, lr=d["lr"], weight_decay=d["weight_decay"], mu=d["momentum"],
                         ns_steps=d["ns_steps"], a=d["a"], b=d["b"], c=d["c"], rms_scale=d["rms_scale"],
                         eps=d["eps"], nesterov=bool(d["nesterov"]), scale_mode=SCALE_MODE_NAMES[d.get("scale_mode", 0)],
                         hidden_size=d.get("hidden_size") or None, schedule=d.get("coeff_schedule"))


def rel_fro(x: np.ndarray, ref: np.ndarray) -> float:
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(x - ref) / den) if den > 0 else float(np.linalg.norm(x))


# Localised checks of O.  One whole-matrix norm would hide a wrong 32 x 32 MFMA sub-tile of a large matrix (0.8 % of
# the norm at 4096 x 4096), so the error is also measured per BLOCK x BLOCK block of the output and per element:
#  * per block: ||dO_blk||_F / max(||O_blk||_F, average block norm) <= BLOCK_FACTOR * tol.  Rounding errors of the
#    iteration are spread over all entries (they live in singular directions, which are dense), so a block's relative
#    error is the matrix's, within sampling noise; measured ratios block / whole are 1.0-1.45.  A 32 x 32 sub-tile that
#    is garbage (100 % error on 1/16 of a block) gives 0.25, twelve times the 2e-2 bar and six times this one.
#  * per element: |dO_ij| <= ELEM_FACTOR * tol * max(|O_ij|, RMS(O)).  For errors of standard deviation tol * RMS(O) the
#    largest of 1e8 entries is below 6 standard deviations; entries far above the RMS (gradient outliers put a few
#    there) carry an error in proportion; a wrong element is off by about max(|O_ij|, RMS(O)) itself.
BLOCK = 128
BLOCK_FACTOR = 2.0
ELEM_FACTOR = 8.0


def block_errors(x: np.ndarray, ref: np.ndarray) -> dict:
    """Largest per-block relative Frobenius error (blocks of BLOCK x BLOCK, ragged edges included; the denominator is
    never below the average block norm, so that a block of tiny entries does not inflate it) and largest elementwise
    error in units of max(|ref_ij|, RMS(ref))."""
    a, b = ref.shape
    d2, r2 = (x - ref) ** 2, ref ** 2
    rows = np.arange(0, a, BLOCK)
    cols = np.arange(0, b, BLOCK)
    d_blk = np.add.reduceat(np.add.reduceat(d2, rows, axis=0), cols, axis=1)
    r_blk = np.add.reduceat(np.add.reduceat(r2, rows, axis=0), cols, axis=1)
    cnt = np.diff(np.append(rows, a))[:, None] * np.diff(np.append(cols, b))[None, :]
    mean_sq = r2.sum() / max(a * b, 1)
    den = np.sqrt(np.maximum(r_blk, mean_sq * cnt))
    rms = np.sqrt(mean_sq)
    if rms == 0.0:
        return {"o_blk_max": float(np.sqrt(d_blk).max()), "o_elem_max": float(np.sqrt(d2.max()))}
    return {"o_blk_max": float((np.sqrt(d_blk) / den).max()),
            "o_elem_max": float((np.abs(x - ref) / np.maximum(np.abs(ref), rms)).max())}


def momentum_error(m_gpu: np.ndarray, m_ref: np.ndarray, m0: np.ndarray, g0: np.ndarray, mu: float) -> float:
    """max |M_gpu - M_ref| / (|mu M0| + |G|): the forward-error scale of one fp32 fused multiply-add."""
    den = np.abs(mu * m0) + np.abs(g0)
    mask = den > 0
    if not mask.any():
        return float(np.max(np.abs(m_gpu - m_ref)))
    return float(np.max(np.abs(m_gpu - m_ref)[mask] / den[mask]))


def bf16_round(x64: np.ndarray) -> np.ndarray:
    """fp64 -> bf16 (round to nearest even) -> fp64, done on the integer bit pattern of the fp32 value."""
    f = x64.astype(np.float32)
    u = f.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def bf16_ulp(x64: np.ndarray) -> np.ndarray:
    e = np.floor(np.log2(np.maximum(np.abs(x64), 1e-38)))
    return 2.0 ** (e - 7)


def check_weight_update(w_gpu: torch.Tensor, w0: np.ndarray, o_gpu: np.ndarray, d) -> dict:
    """Apply stage alone: feed the library's own O to the oracle's update rule and compare W."""
    mode = SCALE_MODE_NAMES[d.get("scale_mode", 0)]
    ref = orc.apply_update(w0, o_gpu, d["lr"], d["weight_decay"], d["rms_scale"], mode, d.get("hidden_size") or None)
    got = to64(w_gpu)
    factor = orc.update_factor(o_gpu, w0.shape, d["rms_scale"], mode, d.get("hidden_size") or None)
    scale = np.abs(w0) * (1 + abs(d["lr"] * d["weight_decay"])) + abs(d["lr"] * factor) * np.abs(o_gpu)
    if w_gpu.dtype == torch.float32:
        err = np.abs(got - ref) / np.maximum(scale, 1e-300)
        return {"max_rel": float(err.max()), "frac_off": 0.0}
    # bf16 weights: the library rounds an fp32 value v once (to nearest even), and v is within the fp32 forward error
    # TOL_ELEM * scale of the exact result, so |got - exact| <= ulp/2 + TOL_ELEM * scale, with the ulp of the binade
    # the rounding lands in.  The second term only matters where the update cancels most of the weight.  Against the
    # fp64 result rounded to bf16 the library may therefore differ, by one ulp, on a small fraction (double rounding).
    ref_b = bf16_round(ref)
    bound = 0.5 * np.maximum(bf16_ulp(ref), bf16_ulp(got)) + TOL_ELEM * scale
    return {"max_excess": float((np.abs(got - ref) / np.maximum(bound, 1e-300)).max()),
            "frac_off": float(np.mean(np.abs(got - ref_b) > 0))}


def run_and_compare(wl: workloads.Workload, device, check=None, steps: int = 1, hp_over=None, max_ws: int = 0,
                    want_rms: bool = False):
    """Runs `steps` library steps over the whole workload and the oracle over the matrices in `check`
    (default: all).  Returns a list of per-(step, matrix) error records."""
    tensors = workloads.make_all(wl, device)
    n = len(tensors)
    check = list(range(n)) if check is None else list(check)
    hp, d = hp_from(wl.hyper, **(hp_over or {}))
    st = binding.MuonStepper(tensors, ns_dtype=wl.ns_dtype, max_workspace_bytes=max_ws)
    host = {i: [to64(t) for t in tensors[i]] for i in check}     # W, G, M before the step
    rms = torch.zeros(n, dtype=torch.float32, device=device) if want_rms else None
    out = []
    for s in range(steps):
        if s > 0:
            for i in range(n):
                g = workloads.make_gradient(wl, i, s, device)
                tensors[i][1].copy_(g)
                if i in host:
                    host[i][1] = to64(g)
        st.step(hp, update_rms=rms)
        torch.cuda.synchronize()
        for i in check:
            w0, g0, m0 = host[i]
            W, M, O = oracle_step(w0, g0, m0, d)
            o_gpu = to64(st.read_update(i))
            m_gpu = to64(tensors[i][2])
            rec = {"step": s, "index": i, "shape": tuple(w0.shape),
                   "o_rel_fro": rel_fro(o_gpu, O), **block_errors(o_gpu, O),
                   "m_err": momentum_error(m_gpu, M, m0, g0, d["momentum"]),
                   "w": check_weight_update(tensors[i][0], w0, o_gpu, d),
                   "o_finite": bool(np.isfinite(o_gpu).all())}
            if want_rms:
                rec["rms_gpu"] = float(rms[i].item())
                rec["rms_ref"] = orc.update_rms(o_gpu)
            out.append(rec)
            # carry the library's own state forward so that each step is compared on identical inputs
            host[i] = [to64(tensors[i][0]), host[i][1], m_gpu]
    st.close()
    return out
