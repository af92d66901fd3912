"""The output layer's entry point that allocates nothing (its per-workgroup candidates live in a static device
array of the library) against the entry point that takes a workspace: same tokens and max logits bit for bit,
on two calls in a row, the second with a smaller input, so that whatever the first call left in the array
must not matter.  The workspace entry point itself is pinned to the oracle in test_gpu_parity.py."""
import numpy as np
import pytest
import torch

import oracle
import workloads
import paper_1805_12096_amd as mq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def run_both(Hd, E):
    M, d = Hd.shape
    V = E.shape[0]
    pe = mq.prepare_weight(dev(E), 8)
    qp = torch.empty(mq.mq_packed_bytes(8, M, d), dtype=torch.uint8, device=DEV)
    s = torch.empty(1, dtype=torch.float32, device=DEV)
    qws = torch.empty(mq.mq_quantize_absmax_ws_bytes(), dtype=torch.uint8, device=DEV)
    mq.mq_quantize_absmax_pack_f32(dev(Hd), M, d, 8, qp, s, qws, qws.numel())
    nws = mq.mq_argmax_ws_bytes(M, V)
    ws = torch.empty(nws, dtype=torch.uint8, device=DEV)
    tok_w = torch.full((M,), -1, dtype=torch.int32, device=DEV)
    val_w = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
    mq.mq_gemm_argmax_packed(qp, pe.packed, M, V, d, s, pe.scale, tok_w, val_w, ws, nws)
    tok_s = torch.full((M,), -1, dtype=torch.int32, device=DEV)
    val_s = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
    mq.mq_gemm_argmax_packed_static(qp, pe.packed, M, V, d, s, pe.scale, tok_s, val_s)
    torch.cuda.synchronize()
    return (tok_w.cpu().numpy(), val_w.cpu().numpy()), (tok_s.cpu().numpy(), val_s.cpu().numpy())


def test_static_scratch_output_layer_two_calls_second_smaller():
    assert torch.cuda.is_available()
    mq.load_library()
    # first call: more rows than one pass of the kernel takes (two passes reuse the array) and the full vocabulary
    c = workloads.config3(M=500, V=36000, d=512)
    (tw, vw), (ts, vs) = run_both(c["Hd"], c["E"])
    assert np.array_equal(ts, tw) and np.array_equal(vs, vw)
    o = oracle.greedy_output_layer(c["Hd"], c["E"])
    assert np.array_equal(ts, o["tok"]) and np.array_equal(vs, o["maxlogit"])
    # second call: fewer rows, fewer words, shorter K -- fewer workgroups and columns of the array are in use
    c2 = workloads.config3(M=37, V=1000, d=192)
    (tw, vw), (ts, vs) = run_both(c2["Hd"], c2["E"])
    assert np.array_equal(ts, tw) and np.array_equal(vs, vw)
    o = oracle.greedy_output_layer(c2["Hd"], c2["E"])
    assert np.array_equal(ts, o["tok"]) and np.array_equal(vs, o["maxlogit"])
    # and the first size once more after the small one
    (tw, vw), (ts, vs) = run_both(c["Hd"], c["E"])
    assert np.array_equal(ts, tw) and np.array_equal(vs, vw)


def test_static_scratch_entry_rejects_what_it_cannot_serve():
    x = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    f = torch.ones(1, dtype=torch.float32, device=DEV)
    t = torch.zeros(8, dtype=torch.int32, device=DEV)
    v = torch.zeros(8, dtype=torch.float32, device=DEV)
    with pytest.raises(mq.MqError) as e:
        mq.mq_gemm_argmax_packed_static(x, x, 24577, 64, 64, f, f, t, v)      # more rows than the limit
    assert e.value.status == 8 and "static scratch" in str(e.value)
    with pytest.raises(mq.MqError) as e:
        mq.mq_gemm_argmax_packed_static(x, x, 8, 64, 1024, f, f, t, v)        # K beyond the streaming kernel
    assert e.value.status == 6
