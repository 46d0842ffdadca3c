"""Helpers for the GPU parity tests: run the HIP path through the C ABI, run the oracle."""
import numpy as np
import torch

from oracle import c_oracle
from paper_2311_03285_amd import slora, synth
from paper_2311_03285_amd.harness import DeviceWorkload, bits_to_device

REL_L2_BAR = 1e-3      # spec tolerance: relative L2 error of the outputs
MAX_ABS_BAR = 1e-2     # spec tolerance: largest absolute error
# what fp32 accumulation of <= 8192 + 128 products of 16-bit values should reach in practice
REL_L2_EXPECTED = 2e-6


def oracle_slot(w: synth.Workload, slot: int, ids=None, x_bits=None, y_in=None):
    """fp64 oracle output for one slot, on a compact re-paging of the adapters the batch uses
    (the oracle's result does not depend on page placement; its own tests pin that)."""
    ids = w.ids if ids is None else np.asarray(ids, dtype=np.int32)
    used = np.unique(ids[ids >= 0])
    rows, lists = w.compact_pool(slot, used)
    if rows.shape[0] == 0:
        rows = np.zeros((1, w.H), dtype=np.uint16)
    x_bits = w.x_bits(slot) if x_bits is None else x_bits
    y_in = w.y_in(slot) if y_in is None else y_in
    return c_oracle.lora_apply(rows, w.dtype, lists, ids, x_bits, y_in)


def gpu_slot(dw: DeviceWorkload, slot: int, plan=None, x_bits=None, y_in=None, stream=None):
    w = dw.w
    plan = dw.plan() if plan is None else plan
    x = bits_to_device(w.x_bits(slot) if x_bits is None else x_bits, dw.device)
    y = torch.from_numpy(np.ascontiguousarray(w.y_in(slot) if y_in is None else y_in)).to(dw.device)
    slora.lora_apply(plan, slot, x.data_ptr(), y.data_ptr(), stream)
    torch.cuda.synchronize(dw.device)
    return y.cpu().numpy()


def errors(got: np.ndarray, ref: np.ndarray):
    d = got.astype(np.float64) - ref
    den = np.linalg.norm(ref)
    return (np.linalg.norm(d) / den if den > 0 else np.linalg.norm(d)), float(np.abs(d).max()) if d.size else 0.0


def assert_close(got, ref, what="", rel_bar=REL_L2_BAR):
    assert np.isfinite(got).all(), f"{what}: non-finite output (a canary page was read?)"
    rel, mx = errors(got, ref)
    assert rel <= rel_bar and mx <= MAX_ABS_BAR, f"{what}: rel-L2 {rel:.3e}, max-abs {mx:.3e}"
    return rel, mx
