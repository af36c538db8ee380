"""The loss entry point that allocates nothing (ftp_softmax_ce_static: its per-row losses live in a file-scope device
array) against ftp_stage_loss, through the C ABI: same loss and same logits gradient, bit for bit, on two calls in a
row, the second on a smaller input; sizes beyond the array are refused."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def stage_loss_reference(P, torch, dtype, batch, classes, logits, labels):
    """(loss, dlogits) of ftp_stage_loss + ftp_stage_backward on a stage that holds only the loss unit."""
    B = P.binding
    units = [dict(kind=B.UNIT_FC, cin=8, cout=classes), dict(kind=B.UNIT_LOSS, cin=classes, cout=classes)]
    model = P.model_create(units, 1, 1, 8, P.F32 if dtype == "f32" else P.BF16)
    stage = P.stage_create(model, 1, 2, batch, 1)
    try:
        sp = torch.cuda.current_stream().cuda_stream
        loss = torch.zeros(1, dtype=torch.float32, device="cuda")
        d = torch.full_like(logits, float("nan"))
        P.stage_forward(stage, 0, logits, None, sp)
        P.stage_loss(stage, 0, labels, loss, sp)
        P.stage_backward(stage, 0, None, d, sp)
        torch.cuda.synchronize()
        return loss.clone(), d
    finally:
        P.stage_destroy(stage)
        P.model_destroy(model)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_static_loss_matches_stage_loss_on_two_calls_in_a_row(dtype):
    import torch
    import paper_2110_02781_amd as P
    from oracle import layers as L
    tdt = torch.float32 if dtype == "f32" else torch.bfloat16
    sp = torch.cuda.current_stream().cuda_stream
    for call, (batch, classes) in enumerate([(48, 1000), (7, 10)]):      # the second call is the smaller one
        print(f"static loss {dtype} call {call}: batch {batch} classes {classes}", flush=True)
        logits = torch.from_numpy(synth.normal(90 + call, "logits", (batch, classes), std=3.0).astype(np.float32)).cuda().to(tdt)
        labels = torch.from_numpy(synth.labels(90 + call, "labels", batch, classes).astype(np.int32)).cuda()
        loss = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
        d = torch.full_like(logits, float("nan"))
        P.softmax_ce_static(logits, labels, batch, classes, P.F32 if dtype == "f32" else P.BF16, d, loss, sp)
        torch.cuda.synchronize()
        ref_loss, ref_d = stage_loss_reference(P, torch, dtype, batch, classes, logits, labels)
        assert torch.equal(loss, ref_loss), (float(loss), float(ref_loss))
        assert torch.equal(d, ref_d)
        # and both against the oracle's definition on the values the kernels saw
        lo, do = L.softmax_ce(logits.float().cpu().numpy().astype(np.float64), labels.cpu().numpy())
        tol = 1e-4 if dtype == "f32" else 2e-2
        assert abs(float(loss) - lo) <= tol * max(1.0, abs(lo))
        assert np.abs(d.float().cpu().numpy() - do).max() <= tol * np.abs(do).max()


def test_static_loss_refuses_what_the_array_cannot_hold():
    import torch
    import paper_2110_02781_amd as P
    t = torch.zeros(16, device="cuda")
    li = torch.zeros(16, dtype=torch.int32, device="cuda")
    with pytest.raises(P.FtpError) as ei:
        P.softmax_ce_static(t, li, P.STATIC_LOSS_MAX_BATCH + 1, 4, P.F32, t, t, None)
    assert ei.value.status == -1 and "beyond" in str(ei.value)
    for bad in (dict(batch=0), dict(classes=0), dict(dtype=7)):
        kw = dict(batch=4, classes=4, dtype=P.F32)
        kw.update(bad)
        with pytest.raises(P.FtpError):
            P.softmax_ce_static(t, li, kw["batch"], kw["classes"], kw["dtype"], t, t, None)
    with pytest.raises(P.FtpError):
        P.softmax_ce_static(None, li, 4, 4, P.F32, t, t, None)
