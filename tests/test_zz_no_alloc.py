"""compactor_compress_static (the entry point that allocates nothing: its scratch is a buffer
inside the library's device image) against compactor_compress, through the C-ABI: same bits on
calls in a row that share the buffer, the later ones smaller than the first."""
import pytest
import torch

from paper_2507_08143_amd import workloads as W
from tests import gpu_util as U

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _say(*a):
    print(*a, flush=True)


def _buffers(C, params, reqs, w):
    so, ko, _ = C.compactor_layout(params, reqs)
    nh = len(reqs) * w.layers * w.kv_heads
    return dict(scores=torch.empty(so[-1], dtype=torch.float32, device=DEV),
                kept_idx=torch.full((ko[-1],), -7, dtype=torch.int32, device=DEV),
                kept_cnt=torch.full((nh,), -7, dtype=torch.int32, device=DEV),
                k_packed=torch.zeros(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                v_packed=torch.zeros(ko[-1], 128, dtype=torch.bfloat16, device=DEV),
                status=torch.full((nh,), -7, dtype=torch.int32, device=DEV))


def _same(a, b, what):
    for name in ("kept_idx", "kept_cnt", "status"):
        assert torch.equal(a[name], b[name]), "%s: %s differs" % (what, name)
    if a["scores"] is not None and b["scores"] is not None:
        assert torch.equal(a["scores"].view(torch.int32), b["scores"].view(torch.int32)), what + ": scores differ"
    for name in ("k_packed", "v_packed"):
        assert torch.equal(a[name].view(torch.int16), b[name].view(torch.int16)), "%s: %s differs" % (what, name)


def _case(C, w, what, scope=0, with_scores=True):
    params, reqs = U.make_call(C, w, DEV)
    params.select_scope = scope
    ref = _buffers(C, params, reqs, w)
    got = _buffers(C, params, reqs, w)
    if not with_scores:
        ref["scores"] = got["scores"] = None
    ws = torch.empty(max(256, C.compactor_workspace_size(params, reqs)), dtype=torch.uint8, device=DEV)
    _say("  %s: %d head-rows, workspace %.1f MB" % (what, w.head_rows, ws.numel() / 1e6))
    C.compactor_compress(params, reqs, workspace=ws, **ref)
    torch.cuda.synchronize()
    C.compactor_compress_static(params, reqs, **got)      # the first call on a device looks the buffer up
    torch.cuda.synchronize()
    free0 = torch.cuda.mem_get_info()[0]
    C.compactor_compress_static(params, reqs, **got)
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free0, "device memory was allocated during the call"
    _same(ref, got, what)
    assert int(ref["status"].max()) == 0
    return params, reqs, ref


def test_static_scratch_compress_equals_compress():
    C = U.binding()
    _say("compress on the static scratch: a large call, then smaller ones on the same buffer")
    # 8 heads of 50000 tokens: selection by several workgroups per head, about 21 MB of scratch
    big = W.config2(DEV, L=2, H=4, n=50000)
    params, reqs, ref = _case(C, big, "2 x 4 heads, n = 50000")
    # the oracle agrees with what both produced (sampled heads)
    st, _ = U.run_and_check(C, big, DEV, heads=[(0, 0, 0), (0, 1, 3)])
    _say("  oracle on 2 heads: max rel err %.3g, swaps %d" % (st["max_rel"], st["swaps"]))
    # smaller, ragged, head-adaptive selection (its histograms live in the same scratch)
    _case(C, W.config4(DEV, L=1, H=3, n_req=3, n_lo=300, n_hi=2500), "ragged batch, layer scope", scope=C.SCOPE_LAYER)
    # smaller still, scores kept inside the scratch
    _case(C, W.config1(DEV, L=1, H=2, n=777, ratio=0.37), "2 heads, n = 777, scores in the scratch", with_scores=False)
    # and the first shape again after the small ones
    got = _buffers(C, params, reqs, big)
    C.compactor_compress_static(params, reqs, **got)
    torch.cuda.synchronize()
    _same(ref, got, "first shape again")


def test_static_scratch_refuses_what_does_not_fit():
    C = U.binding()
    _say("compress on the static scratch: a batch whose scratch exceeds the buffer is refused")
    L, H, n = 64, 80, 16                      # 5120 heads: their first histograms alone take 80 MB
    k = torch.zeros(L, H, n, 128, dtype=torch.bfloat16, device=DEV)
    params = C.Params(L, H, sketch_dim=48, phi=W.make_phi(device=DEV))
    reqs = [C.Request(k_score=k, v_cache=k, ratio=0.5)]
    assert C.compactor_workspace_size(params, reqs) > C.STATIC_SCRATCH_BYTES
    w = W.Workload("too_big", L, H, [W.Request(k, k, 0.5)])
    bufs = _buffers(C, params, reqs, w)
    with pytest.raises(C.CompactorError) as e:
        C.compactor_compress_static(params, reqs, **bufs)
    assert e.value.code == C.EWORKSPACE
    torch.cuda.synchronize()
    assert int(bufs["kept_cnt"].max()) == -7          # nothing was enqueued
    # cut into head groups that fit, the same batch goes through
    params.group_bytes = 256 * n * 256
    C.compactor_compress_static(params, reqs, **bufs)
    torch.cuda.synchronize()
    assert int(bufs["kept_cnt"].min()) == 8
