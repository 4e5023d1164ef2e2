"""vq_gemv_static_workspace (the entry point that allocates nothing) against vq_gemv_with_workspace and the oracle."""
import numpy as np
import pytest

import oracle
import vq_synth as s

pytestmark = pytest.mark.gpu

TOL = 1e-2          # max |y - y_ref| <= TOL * RMS(y_ref): the stated bar of the products


def _run(gpu_lib, torch, L, batch, entry):
    dl = gpu_lib.DeviceLayer(L)
    x_np = s.make_activations(77, L, batch)
    x = torch.from_numpy(x_np).cuda()
    y = torch.full((batch, L.out_features), float("nan"), dtype=torch.float16, device="cuda")
    need = gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch)
    st = torch.cuda.current_stream().cuda_stream
    if entry == "static":
        rc = gpu_lib.vq_gemv_static_workspace(dl.desc, x.data_ptr(), x.stride(0), batch, y.data_ptr(), y.stride(0), st)
    else:
        ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
        rc = gpu_lib.vq_gemv_with_workspace(dl.desc, x.data_ptr(), x.stride(0), batch, y.data_ptr(), y.stride(0), ws.data_ptr(), need, st)
    assert rc == 0, gpu_lib.vq_status_string(rc)
    torch.cuda.synchronize()
    return y.cpu().numpy(), oracle.gemv(L, x_np), need


def test_static_workspace_matches_the_workspace_entry_point_twice_in_a_row(gpu_lib):
    """Two calls in a row, the second on a smaller layer and batch (the library's array keeps the first call's contents):
    each bit-identical to vq_gemv_with_workspace (same kernels, same order of additions) and within the bar of the oracle."""
    import torch
    big = s.make_layer(930, "static_ws_big", 2100, 1560, 6, 4096, 256, 24, 4, 4096, group_vectors=64)     # 5 codebook groups
    small = s.make_layer(931, "static_ws_small", 333, 774, 6, 4096, group_vectors=40)                      # 4 groups, no residual
    for L, batch in ((big, 7), (small, 2)):
        y_static, ref, need = _run(gpu_lib, torch, L, batch, "static")
        assert 0 < need <= gpu_lib.VQ_GEMV_STATIC_WORKSPACE_BYTES
        y_ws, _, _ = _run(gpu_lib, torch, L, batch, "workspace")
        rms = float(np.sqrt((ref ** 2).mean()))
        assert np.abs(y_static.astype(np.float64) - ref).max() <= TOL * rms, L.name
        assert np.array_equal(y_static.view(np.uint16), y_ws.view(np.uint16)), L.name


def test_static_workspace_rejects_what_does_not_fit(gpu_lib):
    import torch
    L = s.make_layer(932, "static_ws_huge", 40000, 1560, 6, 4096, group_vectors=8)          # 33 groups x 16 x 40000 floats > 16 MiB
    dl = gpu_lib.DeviceLayer(L)
    batch = 16
    assert gpu_lib.vq_gemv_workspace_bytes(dl.desc, batch) > gpu_lib.VQ_GEMV_STATIC_WORKSPACE_BYTES
    x = torch.zeros((batch, L.in_features), dtype=torch.float16, device="cuda")
    y = torch.zeros((batch, L.out_features), dtype=torch.float16, device="cuda")
    rc = gpu_lib.vq_gemv_static_workspace(dl.desc, x.data_ptr(), x.stride(0), batch, y.data_ptr(), y.stride(0), None)
    assert rc == gpu_lib.VQ_ERR_WORKSPACE


def test_static_workspace_layer_without_groups_is_plain_gemv(gpu_lib):
    import torch
    L = s.make_layer(933, "static_ws_plain", 150, 1207, 6, 4096, 256)
    y_static, ref, need = _run(gpu_lib, torch, L, 3, "static")
    assert need == 0
    assert np.abs(y_static.astype(np.float64) - ref).max() <= TOL * float(np.sqrt((ref ** 2).mean()))
