"""pc_forward_static: the forward pass for callers that cannot allocate (its workspace is a fixed array inside the
library's device image) against pc_forward, through the C ABI.  Two calls in a row, the second with a smaller batch,
so that whatever the first call left in the shared array must not matter."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import pc_oracle as orc
from paper_2406_00766_amd import binding as pcb
from paper_2406_00766_amd import workloads as W
from tests import tolerances as tol

pytestmark = pytest.mark.gpu


def ll_close(got, ref):
    return np.all(np.abs(got - ref) <= tol.LL_RTOL * np.abs(ref) + tol.LL_ATOL)


def test_forward_static_matches_forward_on_two_calls_in_a_row():
    w = W.reduced(2)                                   # HCLT, K = 32, B = 100 (a ragged tail of 4 columns)
    small = w.with_batch(w.x[:37])
    c = pcb.Circuit(w)
    results = []
    for wb in (w, small):
        print(f"case static forward {wb.name} B={wb.B}", flush=True)
        c.set_batch(wb.x)
        c._ws.fill_(255)
        ref = c.forward().clone()                      # the existing entry point, caller-owned workspace
        assert pcb.pc_workspace_bytes(c.handle, wb.B) <= pcb.PC_STATIC_SCRATCH_BYTES
        ll = torch.full_like(ref, float("nan"))
        pcb.pc_forward_static(c.handle, c.theta, c.tables, c.x, None, wb.B, ll)
        torch.cuda.synchronize()
        assert torch.equal(ll, ref), "same kernels on the same inputs: bit-identical log-likelihoods"
        ref_ll = orc.forward(wb, w.theta, w.tables, wb.x)[1]
        assert ll_close(ll.double().cpu().numpy(), ref_ll)
        results.append(ll.clone())
    assert torch.equal(results[1], results[0][:37])
    # no state is left for the backward pass
    with pytest.raises(pcb.PcError) as e:
        c.backward()
    assert e.value.status_name == "PC_ERR_STATE"
    # with a mask, and a second circuit sharing the same array afterwards
    rng = np.random.default_rng(3)
    mask = (rng.random(small.x.shape) < 0.3).astype(np.uint8)
    c.set_batch(small.x, mask)
    ref = c.forward().clone()
    ll = torch.empty_like(ref)
    pcb.pc_forward_static(c.handle, c.theta, c.tables, c.x, c.mask, small.B, ll)
    torch.cuda.synchronize()
    assert torch.equal(ll, ref)
    w2 = W.reduced(1)
    c2 = pcb.Circuit(w2)
    c2.set_batch(w2.x)
    ref2 = c2.forward().clone()
    ll2 = torch.empty_like(ref2)
    pcb.pc_forward_static(c2.handle, c2.theta, c2.tables, c2.x, None, w2.B, ll2)
    torch.cuda.synchronize()
    assert torch.equal(ll2, ref2)
    c.close(); c2.close()


def test_forward_static_rejects_what_does_not_fit():
    w = W.reduced(3)                                   # 128 hidden states, 40 variables
    c = pcb.Circuit(w)
    B = 1
    while pcb.pc_workspace_bytes(c.handle, B) <= pcb.PC_STATIC_SCRATCH_BYTES:
        B *= 2
    x = torch.zeros((B, w.n_vars), dtype=torch.int32, device="cuda:0")
    ll = torch.empty(B, dtype=torch.float32, device="cuda:0")
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_forward_static(c.handle, c.theta, c.tables, x, None, B, ll)
    assert e.value.status_name == "PC_ERR_WORKSPACE"
    with pytest.raises(pcb.PcError) as e:
        pcb.pc_forward_static(c.handle, c.theta, c.tables, x, None, 0, ll)
    assert e.value.status_name == "PC_ERR_ARG"
    c.close()
