"""C-ABI checks that need no GPU: the library loads, exports every function the headers under
include/ declare, and its host-side logic (argument validation, fixed-point parameters, workspace sizing)
behaves as documented.  No kernel is launched here."""
import ctypes as C
import os
import re

import pytest

import oracle
from paper_2101_07706_amd import csgs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    names = set()
    inc = os.path.join(ROOT, "include")
    for h in sorted(os.listdir(inc)):
        if h.endswith(".h"):
            text = re.sub(r"/\*.*?\*/", "", open(os.path.join(inc, h)).read(), flags=re.S)
            names |= set(re.findall(r"\b(csgs_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_function_is_exported():
    names = declared_functions()
    assert {"csgs_build_probs", "csgs_sample_layer", "csgs_aggregate", "csgs_layer_gemm",
            "csgs_remote_count"} <= set(names)
    L = csgs.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared under include/ but not exported by libcsgs.so"
    # and the binding knows each of them
    assert set(names) <= set(csgs.EXPORTS), set(names) - set(csgs.EXPORTS)


def test_struct_layouts_match_the_header():
    assert C.sizeof(csgs.ProbStats) == 64           # 7 x 8 bytes + 2 x 4
    assert C.sizeof(csgs.Graph) == 56
    assert C.sizeof(csgs.Workspace) == 80 and csgs.Workspace.n_inst.offset == 64 and csgs.Workspace.scan_mode.offset == 68 and csgs.Workspace.inst_stride.offset == 72
    assert C.sizeof(csgs.InstStrides) == 40 and csgs.InstStrides.adj.offset == 8
    assert C.sizeof(csgs.RemoteOut) == 56 and csgs.RemoteOut.remote_total.offset == 24
    assert csgs.Graph.local_lo.offset == 40 and csgs.Graph.rownorm2_max.offset == 48
    assert csgs.Workspace.has_draw.offset == 48 and csgs.Workspace.draw_B.offset == 56


@pytest.mark.parametrize("nS,skew,rmax", [(8192, 16.0, 1.0), (256, 4.0, 1.0), (1, 1.0, 1.0), (3000, 2.5, 1.0),
                                          (8192, 16.0, 4.0), (5, 1.0, 0.25), (100000, 1000.0, 1.0)])
def test_fixed_point_matches_the_oracle_rule(nS, skew, rmax):
    rc, shift, s_fx = csgs.csgs_fixed_point(nS, skew, rmax)
    assert rc == csgs.OK
    assert shift == oracle.shift_for(nS, skew, rmax)
    assert s_fx == round(skew * 16)


def test_fixed_point_rejects():
    assert csgs.csgs_fixed_point(0, 2.0)[0] == csgs.EINVAL
    assert csgs.csgs_fixed_point(10, 0.99)[0] == csgs.EINVAL
    assert csgs.csgs_fixed_point(10, float("nan"))[0] == csgs.EINVAL
    assert csgs.csgs_fixed_point(10, 2.0, 0.0)[0] == csgs.EINVAL
    assert csgs.csgs_fixed_point(2 ** 30, 2.0 ** 20, 1.0)[0] == csgs.ERANGE     # fewer than 24 fraction bits


def test_workspace_sizing():
    b = csgs.csgs_workspace_bytes
    assert b(0, 1, 1, 1) == 0 and b(10, 0, 1, 1) == 0 and b(10, 1, 0, 1) == 0 and b(10, 1, 1, 0) == 0
    small, big = b(1000, 64, 64, 5000), b(2_449_029, 8192, 8192, 127_511_871)
    assert 0 < small < big < 200 * 2 ** 20
    assert small % 256 == 0 and big % 256 == 0
    assert b(1000, 64, 64, 5000) <= b(1000, 128, 64, 5000) <= b(1000, 128, 128, 5000) <= b(1000, 128, 128, 50000)
    assert 0 < csgs.csgs_workspace_clean_bytes(1000) < small


def test_null_arguments_are_rejected_before_any_launch():
    L = csgs.lib()
    z = C.c_void_p(0)
    assert L.csgs_build_probs(None, z, 1, z, 2.0, z, z, z, z, 1, z, None, z, z) == csgs.EINVAL
    assert L.csgs_sample_layer(None, z, 1, z, z, 1, z, 1, 0, 0, z, 0, z, z, z, z, z, z, z, 1, z, None, None, z, z) == csgs.EINVAL
    assert L.csgs_remote_count(z, z, 0, 1, z, 0, z, z, z, z, z) == csgs.EINVAL
    assert L.csgs_aggregate(z, z, z, 1, z, z, z, 1, 1, z, 1, 0, z, 1, 0, 0, z, 1, z) == csgs.EINVAL
    assert L.csgs_layer_gemm(z, 1, 1, z, 1, z, 1, 1, z, 1, z) == csgs.EINVAL
    assert L.csgs_gather_rows(z, 1, 1, 1, 0, z, 1, z, z, 1, z) == csgs.EINVAL
    assert L.csgs_layer_gemm_grad_w(z, 1, z, 1, 1, z, 1, 1, z, 1, z, 0, z) == csgs.EINVAL
    assert L.csgs_layer_gemm_grad_w_static(z, 1, z, 1, 1, z, 1, 1, z, 1, z) == csgs.EINVAL
    assert L.csgs_layer_gemm_grad_z(z, 1, 1, z, 1, z, 1, 1, z, 1, z) == csgs.EINVAL
    assert L.csgs_aggregate_grad(z, z, z, 1, 1, z, 1, z, z, 1, 1, z, 1, z, 1, z, 0, z) == csgs.EINVAL
    assert L.csgs_calib_mfma_f64(z, 1 << 20, 1, 0, z) == csgs.EINVAL
    assert L.csgs_calib_mfma_f64(C.c_void_p(4096), 100, 1, 0, z) == csgs.EINVAL     # sink too small
    assert L.csgs_workspace_init(None, z) == csgs.EINVAL
    ws = csgs.Workspace(0, 0, 10, 1, 1, 1, 0, 0, 0, 0)
    assert L.csgs_workspace_init(C.byref(ws), z) == csgs.EINVAL           # null base


def test_gradient_scratch_sizing():
    w = csgs.csgs_layer_gemm_grad_w_scratch_bytes
    assert w(0, 1, 1) == 0 and w(1, 0, 1) == 0
    assert w(8192, 256, 256) % (256 * 256 * 8) == 0 and 0 < w(8192, 256, 256) <= 64 * 256 * 256 * 8
    assert w(10, 256, 256) == 256 * 256 * 8                     # fewer rows than one K chunk: a single part
    a = csgs.csgs_aggregate_grad_scratch_bytes
    assert a(0, 10) == 0 and a(10, 0) == 0 and 0 < a(8192, 1000) < a(8192, 100000) and a(100, 1000) % 256 == 0


def test_error_strings():
    assert csgs.strerror(csgs.OK) == "ok"
    for code in (csgs.EINVAL, csgs.EWORKSPACE, csgs.EUNSUPPORTED, csgs.ERANGE, csgs.ELAUNCH):
        assert csgs.strerror(code) not in ("ok", "unknown error")
    assert csgs.strerror(-99) == "unknown error"


def test_profile_interface_without_launches():
    L = csgs.lib()
    n = L.csgs_profile_kernel_count()
    names = [L.csgs_profile_kernel_name(k).decode() for k in range(n)]
    assert len(set(names)) == n and "aggregate" in names and "layer_gemm" in names
    assert csgs.csgs_profile_samples() == {}
    assert csgs.csgs_profile_collect() == {}
    assert L.csgs_profile_samples(None, None, 4, None) == csgs.EINVAL


def test_gradient_calls_reject_bad_arguments_before_any_launch():
    L = csgs.lib()
    z, p = C.c_void_p(0), C.c_void_p(4096)       # p: a non-null, aligned address that is never dereferenced on the host
    # scratch too small
    assert L.csgs_layer_gemm_grad_w(p, 8, p, 8, 64, z, 8, 8, p, 8, p, 16, z) == csgs.EWORKSPACE
    assert L.csgs_aggregate_grad(p, p, p, 100, 10, z, 10, z, p, 8, 8, z, 0, p, 8, p, 16, z) == csgs.EWORKSPACE
    # partial sums beyond the static buffer of the form that allocates nothing (checked before anything else runs)
    assert csgs.csgs_layer_gemm_grad_w_scratch_bytes(65536, 2048, 2304) > csgs.GRAD_W_STATIC_BYTES
    assert L.csgs_layer_gemm_grad_w_static(p, 2048, p, 2304, 65536, z, 2048, 2304, p, 2304, z) == csgs.EWORKSPACE
    # leading dimensions below the row width, misaligned scratch
    assert L.csgs_layer_gemm_grad_z(p, 4, 16, z, 8, p, 8, 8, p, 8, z) == csgs.EINVAL
    assert L.csgs_layer_gemm_grad_w(p, 8, p, 8, 64, z, 8, 8, p, 8, C.c_void_p(4100), 1 << 20, z) == csgs.EINVAL
    assert L.csgs_aggregate_grad(p, p, p, 100, 10, z, 10, z, p, 8, 8, z, 0, p, 8, C.c_void_p(4100), 1 << 20, z) == csgs.EINVAL


def test_sampling_calls_reject_workspace_mismatch():
    L = csgs.lib()
    z, p = C.c_void_p(0), C.c_void_p(4096)
    g = csgs.Graph(1000, 5000, 4096, 4096, 4096, 0, 500, 1.0)
    ws = csgs.Workspace(4096, 1 << 30, 1000, 64, 64, 5000, 0, 0, 0, 0)
    st = C.c_void_p(8192)
    # more rows / draws than the workspace was sized for; a graph of another size
    assert L.csgs_build_probs(C.byref(g), p, 65, z, 2.0, p, p, p, z, 1000, p, C.byref(ws), st, z) == csgs.EWORKSPACE
    assert L.csgs_draw_nodes(1000, p, p, 1000, p, 65, 0, 0, z, 0, p, p, p, p, C.byref(ws), st, z) == csgs.EWORKSPACE
    assert L.csgs_draw_nodes(999, p, p, 1000, p, 64, 0, 0, z, 0, p, p, p, p, C.byref(ws), st, z) == csgs.EINVAL
    small = csgs.Workspace(4096, 1024, 1000, 64, 64, 5000, 0, 0, 0, 0)
    assert L.csgs_build_probs(C.byref(g), p, 64, z, 2.0, p, p, p, z, 1000, p, C.byref(small), st, z) == csgs.EWORKSPACE
    # no draw has run on this workspace yet
    assert L.csgs_sampled_adjacency(C.byref(g), p, 10, z, p, p, p, 100, p, C.byref(ws), st, z) == csgs.EINVAL
    # skew below 1, fixed-point range
    assert L.csgs_build_probs(C.byref(g), p, 64, z, 0.5, p, p, p, z, 1000, p, C.byref(ws), st, z) == csgs.EINVAL


def test_instance_descriptors_are_checked():
    """Several instances per call: the count, the stride and the buffer size are checked on the host."""
    L = csgs.lib()
    z, p = C.c_void_p(0), C.c_void_p(4096)
    g = csgs.Graph(1000, 5000, 4096, 4096, 4096, 0, 500, 1.0)
    st = C.c_void_p(8192)
    per = csgs.csgs_workspace_bytes(1000, 64, 64, 5000)

    def probs(ws):
        return L.csgs_build_probs(C.byref(g), p, 65, z, 2.0, p, p, p, z, 1000, p, C.byref(ws), st, z)

    def desc(nbytes, n_inst, stride):
        return csgs.Workspace(4096, nbytes, 1000, 64, 64, 5000, 0, 0, 0, 0, n_inst, 0, stride)

    # (nS = 65 exceeds nS_max, so a descriptor that passes the instance checks ends in EWORKSPACE, before any launch)
    assert probs(desc(4 * per, 4, 1 << 20)) == csgs.EWORKSPACE
    assert L.csgs_workspace_init(C.byref(desc(4 * per - 256, 4, 1 << 20)), z) == csgs.EWORKSPACE   # room for three only
    assert L.csgs_workspace_init(C.byref(desc(4 * per, 4, 0)), z) == csgs.EINVAL                   # no stride
    assert L.csgs_workspace_init(C.byref(desc(4 * per, 4, 1000)), z) == csgs.EINVAL                # not a multiple of 256
    assert L.csgs_workspace_init(C.byref(desc(100 * per, 65, 1 << 20)), z) == csgs.EINVAL          # too many


def test_compute_instance_strides_are_checked():
    L = csgs.lib()
    z, p = C.c_void_p(0), C.c_void_p(4096)
    bad = [csgs.InstStrides(0, 0, 256, 0, 0, 256), csgs.InstStrides(65, 0, 256, 0, 0, 256), csgs.InstStrides(2, 0, 8, 0, 0, 256),
           csgs.InstStrides(2, 0, 256, -16, 0, 256)]
    for inst in bad:
        assert L.csgs_aggregate_n(C.byref(inst), p, p, p, 4, z, z, p, 8, 4, z, 0, 0, z, 8, 0, 0, p, 8, z) == csgs.EINVAL
        assert L.csgs_layer_gemm_n(C.byref(inst), p, 8, 4, z, 8, p, 8, 8, p, 8, z) == csgs.EINVAL
        assert L.csgs_gather_rows_n(C.byref(inst), p, 8, 4, 8, 0, p, 4, z, p, 8, z) == csgs.EINVAL


def test_layer_forward_checks_its_arguments_on_the_host():
    """csgs_layer_forward: which input widths it takes, and what it refuses before anything is enqueued."""
    L = csgs.lib()
    z, p = C.c_void_p(0), C.c_void_p(4096)
    sup = L.csgs_layer_forward_supported
    assert [sup(k, csgs.F32, k, k) for k in (1, 33, 64, 100, 128, 256)] == [1] * 6
    assert [sup(k, csgs.F32, k, k) for k in (0, 65, 101, 130, 258, 300, 512, 602)] == [0] * 8
    assert sup(100, csgs.BF16, 100, 0) == 1 and sup(100, csgs.BF16, 101, 0) == 0 and sup(256, csgs.F32, 256, 258) == 0
    assert sup(64, 7, 64, 64) == 0      # no such element type

    def call(F_in=64, dtype=csgs.F32, ld=64, W=p, ldw=32, H=p, ldh=32, Z=z, ldz=0, adj=p):
        return L.csgs_layer_forward(adj, p, p, 100, z, z, p, ld, 1000, z, 0, 0, z, F_in, dtype, 1, W, ldw, 32, H, ldh, Z, ldz, z)

    assert call(adj=z) == csgs.EINVAL and call(W=z) == csgs.EINVAL and call(H=z) == csgs.EINVAL
    assert call(ld=63) == csgs.EINVAL and call(ldw=31) == csgs.EINVAL and call(ldh=31) == csgs.EINVAL and call(Z=p, ldz=63) == csgs.EINVAL
    assert call(F_in=300, ld=300) == csgs.EUNSUPPORTED and call(F_in=100, ld=101) == csgs.EUNSUPPORTED
    assert call(dtype=7) == csgs.EUNSUPPORTED and call(ldw=1 << 24) == csgs.EUNSUPPORTED
    inst = csgs.InstStrides(3, 0, 16, 16, 0, 16)
    bad = csgs.InstStrides(3, 0, 16, 16, 0, 8)
    args = (p, p, p, 100, z, z, p, 64, 1000, z, 0, 0, z, 64, csgs.F32, 1, p, 32, 32, p, 32, z, 0)
    assert L.csgs_layer_forward_n(C.byref(bad), *args, 0, z) == csgs.EINVAL
    assert L.csgs_layer_forward_n(C.byref(inst), *args, 8, z) == csgs.EINVAL      # stride of Z: a multiple of 16
    assert L.csgs_layer_forward_n(C.byref(inst), *args[:13], 300, *args[14:], 0, z) == csgs.EINVAL   # ld_local below the width
