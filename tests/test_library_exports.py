"""The C-ABI library loads on a machine without a GPU and exports every entry point the
header declares; host-only calls behave; the binding lists the same names."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2408_00232_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_lib(verbose=False)
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "cdf.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cdf_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2408_00232_amd import binding
    names = declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert getattr(lib, n) is not None
    assert sorted(binding.EXPORTS) == names


def test_host_only_calls(lib):
    from paper_2408_00232_amd import binding as B
    assert B.cdf_code_row_bytes(100, 8, B.Q_MINMAX) == 100
    assert B.cdf_code_row_bytes(101, 4, B.Q_MINMAX) == 51
    assert B.cdf_code_row_bytes(7, 8, B.Q_NONE) == 28
    small = B.cdf_workspace_bytes(1000, 128, 10_000)
    big = B.cdf_workspace_bytes(1_000_000, 256, 100_000_000)
    assert 0 < small < big and small % 256 == 0
    # argument validation happens on the host, before any launch
    rc = lib.cdf_cache_filter(None, None, ctypes.c_int32(-1), ctypes.c_int32(4), ctypes.c_int64(4), 0,
                              ctypes.c_float(0.1), 0, None, None, None, None, ctypes.c_size_t(0), None)
    assert rc == B.ERR_INVALID_ARG and b"cdf_cache_filter" in lib.cdf_last_error()
    rc = lib.cdf_quantize(None, None, None, None, ctypes.c_int32(4), ctypes.c_int32(4), ctypes.c_int64(4), 0, 5, 0, 0, 0,
                          None, None, None)
    assert rc == B.ERR_UNSUPPORTED


def test_binding_structs_match_header_layout():
    """Field order of the ctypes argument blocks follows the header's structs."""
    from paper_2408_00232_amd import binding as B
    text = open(os.path.join(ROOT, "include", "cdf.h")).read()
    for name, cls in (("cdf_layer_fwd_args", B.cdf_layer_fwd_args), ("cdf_layer_bwd_args", B.cdf_layer_bwd_args),
                      ("cdf_layer_tf_fwd_args", B.cdf_layer_tf_fwd_args),
                      ("cdf_layer_tf_bwd_args", B.cdf_layer_tf_bwd_args), ("cdf_csr", B.cdf_csr)):
        end = re.search(r"\}\s*" + name + ";", text).start()
        body = text[text.rindex("typedef struct {", 0, end) + len("typedef struct {"):end]
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = []
        for decl in body.split(";"):
            decl = decl.strip()
            if not decl:
                continue
            parts = decl.split(",")
            first = re.findall(r"[A-Za-z_][A-Za-z0-9_]*", parts[0])[-1]
            fields.append(first)
            for extra in parts[1:]:
                fields.append(re.findall(r"[A-Za-z_][A-Za-z0-9_]*", extra)[-1])
        assert fields == [f[0] for f in cls._fields_], name


def test_eps_controller_host_function(lib):
    """The library's controller is host arithmetic: checked here against the hand-worked table."""
    from paper_2408_00232_amd import binding as B
    path = os.path.join(ROOT, "tests", "golden", "eps_controller_cases.txt")
    n = 0
    for line in open(path):
        line = line.split("#")[0].strip()
        if not line:
            continue
        eps, acc, mean, want_eps, want_mean = [float(x) for x in line.split("|")]
        got_eps, got_mean = B.cdf_eps_update(eps, acc, mean)
        assert abs(got_eps - want_eps) < 2e-7 and abs(got_mean - want_mean) < 2e-7, line
        n += 1
    assert n >= 8
    p = B.cdf_eps_params(0.001, 0.02, 0.3, 0.001, 0.01, 1.05, 0.9, 1)
    assert abs(B.cdf_eps_update(0.05, 0.60, 0.50, p)[0] - 0.0525) < 2e-7


def test_new_entry_points_validate_on_the_host(lib):
    """Bad arguments are refused before anything is launched (so this runs without a GPU)."""
    from paper_2408_00232_amd import binding as B
    c32, c64, cf = ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    assert lib.cdf_gather_rows(None, c64(4), None, c32(-1), c32(4), 0, None, c64(4), None) == B.ERR_INVALID_ARG
    assert lib.cdf_gather_rows(None, c64(2), None, c32(3), c32(4), 0, None, c64(4), None) == B.ERR_INVALID_ARG  # ld < dim
    assert lib.cdf_gather_rows(None, c64(4), None, c32(0), c32(4), 0, None, c64(4), None) == B.OK               # no rows
    assert lib.cdf_map_index(None, None, c32(-1), None, None, None) == B.ERR_INVALID_ARG
    assert lib.cdf_map_index(None, None, c32(0), None, None, None) == B.OK
    assert lib.cdf_mark_rows(None, None, c32(5), None, c32(0), None, None) == B.ERR_INVALID_ARG
    assert lib.cdf_relu_fwd(None, None, c64(-1), None) == B.ERR_INVALID_ARG
    assert lib.cdf_relu_fwd(None, None, c64(0), None) == B.OK
    assert lib.cdf_accumulate(None, None, c64(3), None) == B.ERR_INVALID_ARG
    assert lib.cdf_adam_step(None, None, None, None, c64(4), cf(0.01), cf(0.9), cf(0.999), cf(1e-8), c32(0), None) == \
        B.ERR_INVALID_ARG                                                                                      # t starts at 1
    assert lib.cdf_adam_step(None, None, None, None, c64(4), cf(0.01), cf(1.0), cf(0.999), cf(1e-8), c32(1), None) == \
        B.ERR_INVALID_ARG                                                                                      # beta1 = 1
    assert lib.cdf_softmax_xent(None, None, c32(4), c32(0), cf(1.0), None, None, None, None, ctypes.c_size_t(0), None) == \
        B.ERR_INVALID_ARG
    assert lib.cdf_active_rows(None, None, c32(-2), None, None, None, None, ctypes.c_size_t(0), None) == B.ERR_INVALID_ARG
    assert b"cdf_active_rows" in lib.cdf_last_error()


def test_partition_structs_match_header_layout():
    from paper_2408_00232_amd import binding as B
    text = open(os.path.join(ROOT, "include", "cdf.h")).read()
    for name, cls in (("cdf_ebv_params", B.cdf_ebv_params), ("cdf_cut_stats", B.cdf_cut_stats),
                      ("cdf_eps_params", B.cdf_eps_params)):
        end = re.search(r"\}\s*" + name + ";", text).start()
        body = text[text.rindex("typedef struct {", 0, end) + len("typedef struct {"):end]
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = []
        for decl in body.split(";"):
            for part in decl.strip().split(","):
                names = re.findall(r"[A-Za-z_][A-Za-z0-9_]*", part)
                if names:
                    fields.append(names[-1])
        assert fields == [f[0] for f in cls._fields_], name


def test_message_width_limit_is_stated_and_checked_on_the_host(lib):
    """Rows wider than 512 lane-vectors are refused before any launch, by the message calls and by the
    layer steps alike; the limit follows the alignment of width and pitch."""
    from paper_2408_00232_amd import binding as B
    assert B.cdf_max_message_dim(2048, 2048, B.F32) == 2048 and B.cdf_max_message_dim(1024, 1024, B.BF16) == 2048
    assert B.cdf_max_message_dim(602, 602, B.F32) == 1024 and B.cdf_max_message_dim(700, 701, B.F32) == 512
    fake = ctypes.c_void_p(0x1000)            # never dereferenced: the call is refused on the host
    c32, c64 = ctypes.c_int32, ctypes.c_int64
    rc = lib.cdf_quantize(fake, fake, fake, fake, c32(4), c32(2052), c64(2052), 0, 8, 0, 1, 1, fake, fake, None)
    assert rc == B.ERR_UNSUPPORTED and b"too wide" in lib.cdf_last_error()
    rc = lib.cdf_dequantize(fake, fake, fake, fake, c32(4), c32(1026), 8, 0, fake, c64(1026), 0, 1, None)
    assert rc == B.ERR_UNSUPPORTED
    csr = B.cdf_csr(8, 16, 0, 0x1000, 0x1000, 0x1000, None)
    args = B.cdf_layer_fwd_args(ctypes.pointer(csr), 8, 8, 4096, 16, B.F32, 1, 0x1000, 0x1000, 0x1000, 0x1000, 0.05, 0, 8,
                                0, 1, 1, 0x1000, None, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000)
    rc = lib.cdf_gcn_layer_fwd(ctypes.byref(args), None, ctypes.c_size_t(0), None)
    assert rc == B.ERR_UNSUPPORTED and b"wider than the message kernels" in lib.cdf_last_error()


@pytest.mark.timeout(60)
def test_dense_bwd_slab_split_terminates_for_large_weight_matrices(lib):
    """f_in * f_out of 25 M and more: the split of the rows into slabs must still terminate (the call then
    reports the missing workspace; nothing is launched)."""
    from paper_2408_00232_amd import binding as B
    fake = ctypes.c_void_p(0x1000)
    c32, c64 = ctypes.c_int32, ctypes.c_int64
    for n in (1, 1000, 3_000_000):
        rc = lib.cdf_dense_bwd(fake, c64(6144), 0, fake, fake, fake, c32(n), c32(6144), c32(4096), 1, fake, fake, c64(6144),
                               None, ctypes.c_size_t(0), None)
        assert rc == B.ERR_WORKSPACE


def test_spmm_plan_host_checks(lib):
    from paper_2408_00232_amd import binding as B
    assert B.cdf_spmm_plan_bytes(0) == 256 and B.cdf_spmm_plan_bytes(8182) == 512          # 128 chunks of 64 entries
    chunks = (144_515_404 + 1023) // 1024                                                  # 1024 entries per wavefront
    assert B.cdf_spmm_plan_bytes(144_515_404) == (chunks * 4 + 255) // 256 * 256
    csr = B.cdf_csr(8, 16, 100, 0x1000, 0x1000, 0x1000, None)
    assert lib.cdf_spmm_plan(ctypes.byref(csr), ctypes.c_void_p(0x1000), ctypes.c_size_t(4), None) == B.ERR_WORKSPACE
    assert lib.cdf_spmm_plan(None, None, ctypes.c_size_t(0), None) == B.ERR_INVALID_ARG
