"""The C-ABI boundary on the host: exported symbols and argument validation (no GPU work is enqueued)."""
import ctypes
import os
import re

import pytest

import paper_2409_17066_amd as vq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "vq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vq_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = vq.load()
    names = _declared_functions()
    assert set(names) == set(vq.EXPORTED)
    for n in names:
        assert getattr(lib, n) is not None
        assert callable(getattr(vq, n))        # the binding carries the same names


def test_version_and_status_strings():
    assert vq.vq_version() >= 100
    texts = {vq.vq_status_string(s) for s in range(0, -7, -1)}
    assert len(texts) == 7 and vq.vq_status_string(-99) == "unknown status"


def _desc(**kw):
    d = vq.vq_layer_desc(ctypes.sizeof(vq.vq_layer_desc), 8, 30, 6, 256, 0, 0, 0, 0,
                         0x1000, None, None, 0x2000, 16, None, 0, None, 0, None, None)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_valid_descriptor_passes():
    assert vq.vq_validate(_desc()) == vq.VQ_OK
    assert vq.vq_validate(_desc(k_res=16, codebook_res=0x3000, idx_res=0x4000, idx_res_row_stride=16)) == vq.VQ_OK
    assert vq.vq_validate(_desc(n_outlier_cols=8, v_out=4, k_out=16, codebook_out=0x3000, idx_out=0x4000,
                                idx_out_row_stride=16)) == vq.VQ_OK


def test_vectors_down_the_output_dimension_in_the_descriptor():
    assert vq.vq_validate(_desc(orientation=1, idx_row_stride=32)) == vq.VQ_OK
    # outlier columns need not be a multiple of v_out there
    assert vq.vq_validate(_desc(orientation=1, idx_row_stride=32, n_outlier_cols=7, v_out=4, k_out=16, codebook_out=0x3000,
                                idx_out=0x4000, idx_out_row_stride=16)) == vq.VQ_OK


def test_codebook_groups_in_the_descriptor():
    assert vq.vq_validate(_desc(group_vectors=2)) == vq.VQ_OK               # 5 vectors: groups of 2, 2, 1
    assert vq.vq_validate(_desc(group_vectors=1000)) == vq.VQ_OK            # one group
    # the layout that ends with `bias` is still taken, as a layer with one group (whatever follows it in memory)
    old = vq.vq_layer_desc.group_vectors.offset
    assert vq.vq_validate(_desc(struct_size=old, group_vectors=-5)) == vq.VQ_OK


@pytest.mark.parametrize("kw,status", [
    (dict(struct_size=4), vq.VQ_ERR_SHAPE),
    (dict(group_vectors=-1), vq.VQ_ERR_SHAPE),
    (dict(orientation=2), vq.VQ_ERR_SHAPE), (dict(orientation=-1), vq.VQ_ERR_SHAPE),
    (dict(orientation=1, idx_row_stride=16), vq.VQ_ERR_SHAPE),          # 30 indices of 8 bits a stream need 30 bytes
    (dict(out_features=0), vq.VQ_ERR_SHAPE),
    (dict(in_features=0), vq.VQ_ERR_SHAPE),
    (dict(v=0), vq.VQ_ERR_SHAPE), (dict(v=17), vq.VQ_ERR_SHAPE),
    (dict(k=1), vq.VQ_ERR_SHAPE), (dict(k=65537), vq.VQ_ERR_SHAPE),
    (dict(k_res=1), vq.VQ_ERR_SHAPE),
    (dict(codebook=None), vq.VQ_ERR_NULL), (dict(idx=None), vq.VQ_ERR_NULL),
    (dict(codebook=0x1008), vq.VQ_ERR_ALIGNMENT), (dict(idx=0x2004), vq.VQ_ERR_ALIGNMENT),
    (dict(idx_row_stride=0), vq.VQ_ERR_SHAPE),            # 5 vectors x 8 bits need 5 bytes
    (dict(idx_row_stride=24), vq.VQ_ERR_ALIGNMENT),
    (dict(k_res=16), vq.VQ_ERR_NULL),
    (dict(k_res=16, codebook_res=0x3000, idx_res=0x4000, idx_res_row_stride=0), vq.VQ_ERR_SHAPE),
    (dict(n_outlier_cols=7, v_out=4, k_out=16, codebook_out=0x3000, idx_out=0x4000, idx_out_row_stride=16), vq.VQ_ERR_SHAPE),
    (dict(n_outlier_cols=32, v_out=4, k_out=16, codebook_out=0x3000, idx_out=0x4000, idx_out_row_stride=16), vq.VQ_ERR_SHAPE),
    (dict(n_outlier_cols=8, v_out=4, k_out=16), vq.VQ_ERR_NULL),
    (dict(scale=0x5001), vq.VQ_ERR_ALIGNMENT),
])
def test_invalid_descriptors(kw, status):
    assert vq.vq_validate(_desc(**kw)) == status


def test_entry_points_reject_bad_arguments_before_any_launch():
    d = _desc()
    assert vq.vq_validate(None) == vq.VQ_ERR_NULL
    assert vq.vq_dequant(None, 0x9000, 30) == vq.VQ_ERR_NULL
    assert vq.vq_dequant(d, None, 30) == vq.VQ_ERR_NULL
    assert vq.vq_dequant(d, 0x9000, 29) == vq.VQ_ERR_SHAPE
    assert vq.vq_dequant(d, 0x9001, 30) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemv(d, None, 30, 1, 0x9000, 8) == vq.VQ_ERR_NULL
    assert vq.vq_gemv(d, 0x8000, 30, 0, 0x9000, 8) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv(d, 0x8000, 30, 17, 0x9000, 8) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv(d, 0x8000, 28, 1, 0x9000, 8) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv(d, 0x8000, 30, 1, 0x9000, 7) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv(d, 0x8001, 30, 1, 0x9000, 8) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemv(d, 0x8000, 30, 1, 0x9001, 8) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemm(d, 0x8000, 32, 0, 0x9000, 8) == vq.VQ_ERR_SHAPE        # empty token batch
    assert vq.vq_gemm(d, 0x8000, 30, 4, 0x9000, 8) == vq.VQ_ERR_ALIGNMENT    # ldx not a multiple of 8
    assert vq.vq_gemm(d, 0x8008, 32, 4, 0x9000, 8) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemm(d, None, 32, 4, 0x9000, 8) == vq.VQ_ERR_NULL
    assert vq.vq_gemm_workspace_bytes(_desc(v=0), 4) == 0


def test_gemv_multi_rejects_bad_arguments_before_any_launch():
    d, e = _desc(), _desc(out_features=5)
    ok = dict(x_ptr=0x8000, ldx=30, batch=1, y_ptrs=[0x9000, 0xA000], ldys=[8, 5])
    assert vq.vq_gemv_multi([d, e], **dict(ok, x_ptr=None)) == vq.VQ_ERR_NULL
    assert vq.vq_gemv_multi([d, e], **dict(ok, y_ptrs=[0x9000, None])) == vq.VQ_ERR_NULL
    assert vq.vq_gemv_multi([d, e], **dict(ok, batch=0)) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([d, e], **dict(ok, batch=17)) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([d, e], **dict(ok, ldys=[8, 4])) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([d, e], **dict(ok, ldx=29)) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([d, e], **dict(ok, y_ptrs=[0x9000, 0xA001])) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemv_multi([d, _desc(in_features=36, idx_row_stride=16)], **ok) == vq.VQ_ERR_SHAPE     # not the same activations
    assert vq.vq_gemv_multi([d, _desc(v=0)], **ok) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([d] * 9, 0x8000, 30, 1, [0x9000] * 9, [8] * 9) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_multi([], 0x8000, 30, 1, [], []) == vq.VQ_ERR_SHAPE


def test_gemv_with_workspace_rejects_bad_arguments_before_any_launch():
    d = _desc()
    assert vq.vq_gemv_workspace_bytes(d, 4) == 0                       # one group: no kernel would use a workspace
    assert vq.vq_gemv_workspace_bytes(_desc(v=0), 4) == 0
    assert vq.vq_gemv_with_workspace(d, None, 30, 1, 0x9000, 8) == vq.VQ_ERR_NULL
    assert vq.vq_gemv_with_workspace(d, 0x8000, 30, 17, 0x9000, 8) == vq.VQ_ERR_SHAPE
    assert vq.vq_gemv_with_workspace(d, 0x8000, 30, 1, 0x9001, 8) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_gemv_with_workspace(d, 0x8000, 30, 1, 0x9000, 8, 0xA010, 4096) == vq.VQ_ERR_ALIGNMENT
    big = _desc(in_features=6 * 64, idx_row_stride=96, v=6, k=4096, group_vectors=16)
    assert vq.vq_gemv_workspace_bytes(big, 2) >= 4 * (2 * 8 + 16) * 4   # 4 groups x (2 tokens x 8 rows + 16 activation sums)
    # groups that do not start on a dword of the index stream: not the matrix-core kernel's, but the kernel that keeps one table
    # in LDS at a time takes a group per workgroup too (6 groups x (2 x 8 + 16) sums)
    assert vq.vq_gemv_workspace_bytes(_desc(in_features=6 * 64, idx_row_stride=96, v=6, k=4096, group_vectors=12), 2) >= 6 * (2 * 8 + 16) * 4
    assert vq.vq_gemv_workspace_bytes(_desc(in_features=5 * 64, idx_row_stride=96, v=5, k=4096, group_vectors=12), 2) == 0    # no kernel of v = 5 uses one


def test_gemv_workspace_for_vectors_down_the_output_dimension():
    """Orientation 1 on the matrix cores cuts the columns into parts when a workspace is there: asked for from two rows
    on (one row stays on the kernel that needs none), sized parts x (rows x tokens + 16) floats, parts >= 2."""
    d = _desc(orientation=1, out_features=96, in_features=1024, idx_row_stride=1536, v=6, k=4096)
    assert vq.vq_validate(d) == vq.VQ_OK
    assert vq.vq_gemv_workspace_bytes(d, 1) == 0
    for batch in (2, 5, 16):
        need = vq.vq_gemv_workspace_bytes(d, batch)
        assert need >= 2 * (batch * 96 + 16) * 4 and need % 256 == 0, batch
    # streams too short to cut (a part needs a 32-column window per wave), odd numbers of outlier columns: no workspace
    assert vq.vq_gemv_workspace_bytes(_desc(orientation=1, out_features=96, in_features=256, idx_row_stride=384, v=6, k=4096), 4) == 0
    odd = _desc(orientation=1, out_features=96, in_features=1024 + 7, idx_row_stride=1536, v=6, k=4096, n_outlier_cols=7, v_out=4, k_out=16,
                codebook_out=0x3000, idx_out=0x4000, idx_out_row_stride=16)
    assert vq.vq_validate(odd) == vq.VQ_OK and vq.vq_gemv_workspace_bytes(odd, 4) == 0
    # codebook groups are parts by themselves, from one row on
    grouped = _desc(orientation=1, out_features=96, in_features=1024, idx_row_stride=1536, v=6, k=4096, group_vectors=256)
    assert vq.vq_gemv_workspace_bytes(grouped, 1) >= 4 * (96 + 16) * 4
    # so is a row too long for the one-row kernel's LDS (28672 activations beside two 64 KB tables)
    long_rows = _desc(orientation=1, out_features=96, in_features=28672, idx_row_stride=43008, v=6, k=4096, k_res=4096,
                      codebook_res=0x5000, idx_res=0x6000, idx_res_row_stride=43008)
    assert vq.vq_validate(long_rows) == vq.VQ_OK
    assert vq.vq_gemv_workspace_bytes(long_rows, 1) >= 2 * (96 + 16) * 4


def test_assign_rejects_bad_arguments_before_any_launch():
    ok = dict(W_ptr=0x8000, B_ptr=None, ld=30, rows=8, cols=30, codebook_ptr=0x1000, v=6, k=256, idx_ptr=0x2000, idx_row_stride=16)
    assert vq.vq_assign(**dict(ok, W_ptr=None)) == vq.VQ_ERR_NULL
    assert vq.vq_assign(**dict(ok, codebook_ptr=None)) == vq.VQ_ERR_NULL
    assert vq.vq_assign(**dict(ok, idx_ptr=None)) == vq.VQ_ERR_NULL
    for bad in (dict(rows=0), dict(cols=0), dict(ld=29), dict(v=0), dict(v=17), dict(k=1), dict(k=65537)):
        assert vq.vq_assign(**dict(ok, **bad)) == vq.VQ_ERR_SHAPE, bad
    assert vq.vq_assign(**dict(ok, cols=30, k=4096, idx_row_stride=0)) == vq.VQ_ERR_SHAPE       # 5 x 12 bits need 8 bytes
    assert vq.vq_assign(**dict(ok, W_ptr=0x8001)) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_assign(**dict(ok, B_ptr=0x8001)) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_assign(**dict(ok, idx_ptr=0x2008)) == vq.VQ_ERR_ALIGNMENT
    assert vq.vq_assign(**dict(ok, idx_row_stride=24)) == vq.VQ_ERR_ALIGNMENT


def test_assign_down_rejects_bad_arguments_before_any_launch():
    ok = dict(W_ptr=0x8000, B_ptr=None, ld=30, rows=8, cols=30, codebook_ptr=0x1000, v=6, k=256, idx_ptr=0x2000, idx_row_stride=32)
    assert vq.vq_assign_down(**dict(ok, W_ptr=None)) == vq.VQ_ERR_NULL
    for bad in (dict(rows=0), dict(cols=0), dict(ld=29), dict(v=17), dict(k=1)):
        assert vq.vq_assign_down(**dict(ok, **bad)) == vq.VQ_ERR_SHAPE, bad
    assert vq.vq_assign_down(**dict(ok, idx_row_stride=16)) == vq.VQ_ERR_SHAPE         # 30 indices of 8 bits a stream
    assert vq.vq_assign_down(**dict(ok, idx_ptr=0x2004)) == vq.VQ_ERR_ALIGNMENT


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2409_17066_amd", "__init__.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
