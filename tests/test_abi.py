"""Host-side checks of the C ABI: the built library loads, exports every function the header declares, and
rejects bad arguments before anything is launched (so these calls are safe without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "moe_layer.h")
LIB = os.path.join(ROOT, "paper_2602_03495_amd", "libmoe_mi355x.so")

MOE_OK, MOE_EINVAL, MOE_EUNSUPPORTED, MOE_ELAUNCH, MOE_EWORKSPACE = 0, -1, -2, -3, -4


class Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("T", "d", "N", "k", "I", "ffn_path", "weight_layout")]


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    return C.CDLL(LIB)


def test_header_declares_the_four_named_calls():
    names = declared_functions()
    for n in ("moe_route", "moe_predict_workload", "moe_expert_ffn", "moe_combine", "moe_workspace_bytes",
              "moe_strerror", "moe_dense_route", "moe_shared_gate", "moe_pack_weights", "moe_expert_ffn_stage"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_lists_the_same_symbols():
    from paper_2602_03495_amd import binding
    assert sorted(binding.EXPORTS) == declared_functions()
    assert C.sizeof(binding.MoeShape) == 28 == C.sizeof(Shape)


def test_strerror(lib):
    lib.moe_strerror.restype = C.c_char_p
    assert lib.moe_strerror(0) == b"ok"
    for code in (MOE_EINVAL, MOE_EUNSUPPORTED, MOE_ELAUNCH, MOE_EWORKSPACE, -99):
        assert len(lib.moe_strerror(code)) > 0


def test_workspace_bytes_and_shape_validation(lib):
    n = C.c_size_t(0)
    good = Shape(2048, 4096, 8, 2, 14336, 0)
    assert lib.moe_workspace_bytes(C.byref(good), C.byref(n)) == MOE_OK
    R = 2048 * 2
    assert n.value >= R * 14336 * 2           # room for the inner activations
    assert n.value < 2 * R * 14336 * 2
    assert lib.moe_workspace_bytes(C.byref(good), None) == MOE_EINVAL
    assert lib.moe_workspace_bytes(None, C.byref(n)) == MOE_EINVAL
    for bad in (Shape(0, 4096, 8, 2, 14336, 0),      # no tokens
                Shape(16, 4096, 8, 9, 14336, 0),     # k > N
                Shape(16, 4096, 8, 0, 14336, 0),     # k < 1
                Shape(16, 4096, 129, 2, 14336, 0),   # too many experts
                Shape(16, 4096, 64, 9, 14336, 0),    # k above the supported maximum
                Shape(16, 4100, 8, 2, 14336, 0),     # d not a multiple of 128
                Shape(16, 16384, 8, 2, 14336, 0),    # d too large
                Shape(16, 4096, 8, 2, 160, 0)):      # I not a multiple of 128
        assert lib.moe_workspace_bytes(C.byref(bad), C.byref(n)) == MOE_EINVAL


def test_entry_points_reject_null_and_misaligned_pointers_before_launching(lib):
    s = Shape(16, 256, 8, 2, 512, 0)
    p = C.c_void_p(0x1000)        # never dereferenced: validation fails first
    z = C.c_void_p(0)
    assert lib.moe_route(C.byref(s), z, p, z, 1, p, p, p, p, p, p, p, z) == MOE_EINVAL
    assert lib.moe_route(C.byref(s), p, p, z, 7, p, p, p, p, p, p, p, z) == MOE_EINVAL          # bad norm mode
    assert lib.moe_route(C.byref(s), C.c_void_p(0x1004), p, z, 1, p, p, p, p, p, p, p, z) == MOE_EINVAL
    assert lib.moe_predict_workload(C.byref(s), p, p, p, z, 0, p, p, p, z) == MOE_EINVAL         # p < 1
    assert lib.moe_predict_workload(C.byref(s), p, p, p, z, 9, p, p, p, z) == MOE_EINVAL         # p > N
    assert lib.moe_predict_workload(C.byref(s), p, z, p, z, 2, p, p, p, z) == MOE_EINVAL         # no res_vec
    assert lib.moe_predict_workload(C.byref(s), p, p, p, z, 2, p, p, C.c_void_p(0x1010), z) == MOE_EWORKSPACE
    assert lib.moe_expert_ffn(C.byref(s), p, p, p, p, p, p, z, z, p, p, z) == MOE_EINVAL          # no w2
    assert lib.moe_expert_ffn(C.byref(s), p, p, p, p, p, p, p, z, p, C.c_void_p(0x1010), z) == MOE_EWORKSPACE
    bad_path = Shape(16, 256, 8, 2, 512, 5, 1)
    assert lib.moe_expert_ffn(C.byref(bad_path), p, p, p, p, p, p, p, z, p, p, z) == MOE_EINVAL
    skinny_big = Shape(64, 256, 8, 2, 512, 2, 1)  # the skinny path takes at most 16 tokens
    assert lib.moe_expert_ffn(C.byref(skinny_big), p, p, p, p, p, p, p, z, p, p, z) == MOE_EUNSUPPORTED
    assert lib.moe_combine(C.byref(s), p, p, p, p, z, z, 0, z, z, z) == MOE_EINVAL                # no out
    assert lib.moe_combine(C.byref(s), p, p, p, p, z, p, 0, z, p, z) == MOE_EINVAL                # shared_y without count
    assert lib.moe_dense_route(C.byref(s), p, p, p, z) == MOE_EINVAL                              # needs k == N
    assert lib.moe_shared_gate(C.byref(s), p, z, p, z) == MOE_EINVAL
    assert lib.moe_pack_weights(8, 500, 256, p, C.c_void_p(0x2000), z) == MOE_EINVAL              # rows not a multiple of 16
    assert lib.moe_pack_weights(8, 512, 250, p, C.c_void_p(0x2000), z) == MOE_EINVAL              # K not a multiple of 32
    assert lib.moe_pack_weights(8, 512, 256, p, p, z) == MOE_EINVAL                               # in place


def test_new_entry_points_reject_bad_arguments_before_launching(lib):
    s = Shape(16, 256, 8, 2, 512, 0)
    p = C.c_void_p(0x1000)
    z = C.c_void_p(0)
    lib.moe_res_vec_workspace_bytes.restype = C.c_size_t
    assert lib.moe_res_vec_workspace_bytes(256) >= 64 * 256 * 8
    assert lib.moe_res_vec_workspace_bytes(0) == 0
    assert lib.moe_res_vec_accumulate(10, 250, p, p, p, p, z) == MOE_EINVAL       # d not a multiple of 8
    assert lib.moe_res_vec_accumulate(-1, 256, p, p, p, p, z) == MOE_EINVAL
    assert lib.moe_res_vec_accumulate(10, 256, z, p, p, p, z) == MOE_EINVAL       # no h_cur
    assert lib.moe_res_vec_accumulate(10, 256, p, p, z, p, z) == MOE_EINVAL       # no accumulator
    assert lib.moe_res_vec_accumulate(10, 256, p, p, C.c_void_p(0x1004), p, z) == MOE_EINVAL
    assert lib.moe_res_vec_finish(256, p, C.c_int64(0), p, z) == MOE_EINVAL       # empty calibration set
    assert lib.moe_res_vec_finish(256, z, C.c_int64(5), p, z) == MOE_EINVAL
    # moe_route_predict: the union of the two calls' checks, and the workspace is required
    rp = lambda *a: lib.moe_route_predict(C.byref(s), *a)
    assert rp(p, p, z, 1, p, p, p, p, p, p, p, p, z, 2, p, p, z, z) == MOE_EINVAL            # no workspace
    assert rp(p, p, z, 1, p, p, p, p, p, p, z, p, z, 2, p, p, p, z) == MOE_EINVAL            # no res_vec
    assert rp(p, p, z, 1, p, p, p, p, p, p, p, p, z, 9, p, p, p, z) == MOE_EINVAL            # p > N
    assert rp(p, p, z, 3, p, p, p, p, p, p, p, p, z, 2, p, p, p, z) == MOE_EINVAL            # bad norm mode
    assert rp(p, p, z, 1, p, p, p, p, p, p, C.c_void_p(0x1004), p, z, 2, p, p, p, z) == MOE_EINVAL   # res_vec alignment
    assert rp(p, p, z, 1, p, p, p, p, p, p, p, p, z, 2, p, p, C.c_void_p(0x1010), z) == MOE_EWORKSPACE
    assert lib.moe_predict_workload(C.byref(s), p, C.c_void_p(0x1004), p, z, 2, p, p, p, z) == MOE_EINVAL


def test_append_shared_rejects_bad_arguments_before_launching(lib):
    s = Shape(16, 256, 8, 2, 512, 0)
    p = C.c_void_p(0x1000)
    z = C.c_void_p(0)
    ap = lambda n_sh, h, wsg, *tables: lib.moe_append_shared(C.byref(s), n_sh, h, wsg, *tables, z)
    ok = (p,) * 12
    assert ap(0, z, z, *ok) == MOE_EINVAL                                          # no shared expert
    assert ap(7, z, z, *ok) == MOE_EINVAL                                          # k + n_shared > 8 slots
    assert ap(2, z, p, *ok) == MOE_EINVAL                                          # a gate vector without h
    assert ap(2, C.c_void_p(0x1004), p, *ok) == MOE_EINVAL                         # h misaligned
    for i in range(12):                                                            # every table pointer is required
        assert ap(2, z, z, *(ok[:i] + (z,) + ok[i + 1:])) == MOE_EINVAL
    wide = Shape(16, 256, 127, 2, 512, 0)
    assert lib.moe_append_shared(C.byref(wide), 2, z, z, *ok, z) == MOE_EINVAL     # N + n_shared > 128 experts


def test_expert_ffn_refuses_weights_not_declared_as_packed(lib):
    # the kernels read the weights in the fragment order of moe_pack_weights only; the library cannot see which layout
    # an array has, so the shape carries the caller's statement and anything but "packed" is refused before any launch
    # (a zero-initialised shape says row-major).  All other arguments of these calls are valid-looking.
    p, z = C.c_void_p(0x1000), C.c_void_p(0)
    for layout in (0, 2, -1):
        s = Shape(16, 256, 8, 2, 512, 0, layout)
        assert lib.moe_expert_ffn(C.byref(s), p, p, p, p, p, p, p, z, p, p, z) == MOE_EUNSUPPORTED
        assert lib.moe_expert_ffn_stage(C.byref(s), p, p, p, p, p, p, p, z, p, p, 1, z) == MOE_EUNSUPPORTED
        assert lib.moe_expert_ffn_static(C.byref(s), p, p, p, p, p, p, p, z, p, z) == MOE_EUNSUPPORTED
    lib.moe_strerror.restype = C.c_char_p
    assert b"moe_pack_weights" in lib.moe_strerror(MOE_EUNSUPPORTED)
    # the tag is read by the expert-FFN calls only
    n = C.c_size_t(0)
    assert lib.moe_workspace_bytes(C.byref(Shape(16, 256, 8, 2, 512, 0, 0)), C.byref(n)) == MOE_OK


def test_route_shared_rejects_bad_arguments_before_launching(lib):
    s = Shape(16, 256, 8, 2, 512, 0, 1)
    p, z = C.c_void_p(0x1000), C.c_void_p(0)
    call = lambda n_sh, h, wsg, *tables: lib.moe_route_shared(C.byref(s), n_sh, h, p, z, 1, wsg, *tables, p, z)
    ok = (p,) * 12
    assert call(0, p, z, *ok) == MOE_EINVAL                                        # no shared expert
    assert call(7, p, z, *ok) == MOE_EINVAL                                        # k + n_shared > 8 slots
    assert call(2, z, z, *ok) == MOE_EINVAL                                        # h feeds the gate: required
    assert call(2, p, C.c_void_p(0x1004), *ok) == MOE_EINVAL                       # gate vector misaligned
    for i in range(12):                                                            # every table pointer is required
        assert call(2, p, z, *(ok[:i] + (z,) + ok[i + 1:])) == MOE_EINVAL
    assert lib.moe_route_shared(C.byref(s), 2, p, p, z, 5, z, *ok, p, z) == MOE_EINVAL                  # bad norm mode
    assert lib.moe_route_shared(C.byref(s), 2, p, p, z, 1, z, *ok, C.c_void_p(0x1010), z) == MOE_EWORKSPACE
