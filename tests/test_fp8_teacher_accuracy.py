"""Accuracy study of the fp8 teacher head, on the CPU with the fp64 oracle only.

The paper reports that FP8 teacher INFERENCE leaves the student's loss curves unchanged (Table 3 and the
text around it); quantising the teacher's output head and final hidden states as well is this build's
extension, so its effect is measured here: the loss and the gradients obtained from e4m3 teacher operands
(one scale per array) against those from the original bf16 operands, on inputs drawn like the benchmark
workloads.  The numbers are recorded in the assertion bounds (about 4x the observed values)."""
import numpy as np
import pytest

from oracle import kd_oracle as O
from paper_2603_01875_amd import inputs as I
from tests import gpu_util as G


def _rel(a, b):
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


@pytest.mark.parametrize("name,kind,beta,loss_tol,grad_tol", [
    ("fkl_bf16", I.FKL, 0.5, 1e-2, 0.15),        # observed: loss 2.1e-3, gradients 0.03 / 0.04, cosine 0.9992
    ("rkl_bf16", I.RKL, 0.5, 1e-2, 0.15),        #           3.2e-3, 0.03 / 0.04, 0.9994
    ("jsd_bf16", I.JSD, 0.5, 1e-2, 0.15),        #           2.3e-3, 0.04 / 0.04, 0.9991
    ("long_peaked", I.JSD, 0.1, 1e-2, 0.25),     #           0.8e-3, 0.075 / 0.076, 0.9972 (near-one-hot teacher)
])
def test_fp8_teacher_changes_loss_and_gradients_little(name, kind, beta, loss_tol, grad_tol):
    # hidden sizes as in the workload (the quantisation noise of a logit averages over H_t), fewer tokens and
    # a smaller vocabulary so that fp64 finishes in seconds
    w = I.workload(name)
    cfg = I.scaled(w, batch=1, seq=96, V=4096, H_t=min(w.H_t, 2048), H_s=min(w.H_s, 512), mask="ones")
    data = I.generate(cfg)
    f8 = G.fp8_teacher(data)
    ref = O.kd_loss_fwd_bwd(data["h_t"], data["W_t"], data["h_s"], data["W_s"], None, cfg.tau, kind, beta, O.W_VH)
    q = O.kd_loss_fwd_bwd(f8["h_t"], f8["W_t"], data["h_s"], data["W_s"], None, cfg.tau, kind, beta, O.W_VH)
    dl = abs(q["loss"] - ref["loss"]) / ref["loss"]
    dh, dW = _rel(q["grad_h_s"], ref["grad_h_s"]), _rel(q["grad_W_s"], ref["grad_W_s"])
    cos = float((q["grad_W_s"] * ref["grad_W_s"]).sum() /
                (np.linalg.norm(q["grad_W_s"]) * np.linalg.norm(ref["grad_W_s"])))
    print(f"{name}: loss {ref['loss']:.5f} -> {q['loss']:.5f} (rel {dl:.2e}); grad_h_s rel L2 {dh:.3f}, "
          f"grad_W_s rel L2 {dW:.3f}, cosine {cos:.5f}")
    assert dl <= loss_tol
    assert dh <= grad_tol and dW <= grad_tol
    assert cos >= 0.99
