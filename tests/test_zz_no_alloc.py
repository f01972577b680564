"""mxq_tensor_absmax_static -- the entry point for callers that cannot allocate -- through the C
ABI against mxq_tensor_absmax_ws (same kernels, caller-owned workspace) and mxq_tensor_absmax:
bit-identical outputs on two calls in a row, the second on a smaller input with a smaller
maximum (a value left in the library's array by the first call would show), then on more sizes
and both dtypes; the size limit is an error, not a launch."""
import numpy as np
import pytest
import torch

from paper_2605_08565_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_static_workspace_entry_point_matches_the_workspace_one(oracle):
    from paper_2605_08565_amd import mxq
    assert torch.cuda.is_available()
    L = mxq.lib()
    stream = int(torch.cuda.current_stream().cuda_stream)
    ws = mxq.absmax_workspace()
    first = W.config3()                                              # 8192 x 4096 bf16, maximum ~ 250
    second = W.student_t_weights(513, 1000, seed=21)                 # smaller tensor, maximum < 1
    more = [W.bf16_bits_to_f32(first[:300]), W.normal_f32(1, 6, 3) * np.float32(1e-4), np.zeros((2, 8), np.float32),
            W.normal_f32(2049, 4099, 5)]
    tensors = [mxq.from_bits(a) for a in [first, second] + more]
    out_s = torch.full((len(tensors),), -1.0, dtype=torch.float32, device="cuda")
    out_w = torch.full((len(tensors),), -2.0, dtype=torch.float32, device="cuda")
    out_p = torch.full((len(tensors),), -3.0, dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for i, t in enumerate(tensors):                                  # back to back on one stream
        rows, cols = t.shape
        dt = mxq.DT_BF16 if t.dtype == torch.bfloat16 else mxq.DT_F32
        print(f"[no-alloc] call {i} shape={tuple(t.shape)} dtype={t.dtype}", flush=True)
        assert L.mxq_tensor_absmax_static(t.data_ptr(), rows, cols, dt, out_s[i:i + 1].data_ptr(), stream) == mxq.OK
        assert L.mxq_tensor_absmax_ws(t.data_ptr(), rows, cols, dt, out_w[i:i + 1].data_ptr(), ws.data_ptr(),
                                      ws.numel(), stream) == mxq.OK
        assert L.mxq_tensor_absmax(t.data_ptr(), rows, cols, dt, out_p[i:i + 1].data_ptr(), stream) == mxq.OK
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    s, w, p = (o.cpu().numpy().view(np.uint32) for o in (out_s, out_w, out_p))
    assert (s == w).all() and (s == p).all(), (s, w, p)
    want = np.array([oracle.tensor_absmax(a) for a in [first, second] + more], np.float32)
    assert (s == want.view(np.uint32)).all()
    assert want[1] < want[0]
    # empty tensor: writes zero; beyond the stated maximum: refused before any launch
    assert L.mxq_tensor_absmax_static(None, 0, 16, 0, out_s[0:1].data_ptr(), stream) == mxq.OK
    torch.cuda.synchronize()
    assert float(out_s.cpu()[0]) == 0.0
    assert L.mxq_tensor_absmax_static(tensors[0].data_ptr(), 1 << 21, (1 << 19) + 8, 0, out_s[0:1].data_ptr(),
                                      stream) == mxq.ERR_UNSUPPORTED
    assert L.mxq_tensor_absmax_static(tensors[0].data_ptr(), 4, 4, 0, None, stream) == mxq.ERR_INVALID_ARG
    # a second round after the refusals: the array is still in its resting state
    t = tensors[1]
    assert L.mxq_tensor_absmax_static(t.data_ptr(), t.shape[0], t.shape[1], 0, out_s[1:2].data_ptr(), stream) == mxq.OK
    torch.cuda.synchronize()
    assert out_s.cpu().numpy().view(np.uint32)[1] == want.view(np.uint32)[1]
