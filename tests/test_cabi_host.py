"""Host-only checks of the C interface: the shared library loads, exports every function that
include/des.h declares, and rejects bad arguments before touching a device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_1909_04823_amd", "libdes.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libdes.so is not built: run `python -m paper_1909_04823_amd.build`")
    return C.CDLL(LIB)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "des.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(des_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"des_table_create", "des_table_insert", "des_table_find", "des_partial_forward_lr",
            "des_partial_forward_fm", "des_partial_forward_pool", "des_aggregate_partials",
            "des_backward_update_sgd", "des_backward_update_adagrad"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in des.h but not exported"


def test_binding_lists_the_same_entry_points():
    import importlib.util
    spec = importlib.util.find_spec("paper_1909_04823_amd.des")
    src = open(spec.origin).read()
    for n in declared_functions():
        assert n in src, f"binding does not know {n}"


def test_host_side_validation_needs_no_device(lib):
    from paper_1909_04823_amd.des import TableConfig, ERR_INVALID_ARG, OK
    lib.des_status_string.restype = C.c_char_p
    assert lib.des_status_string(3) == b"table full"
    sb, wb = C.c_size_t(), C.c_size_t()
    q = lib.des_table_query_bytes
    q.argtypes = [C.POINTER(TableConfig), C.c_int64, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
    cfg = TableConfig()
    cfg.dim, cfg.capacity_rows, cfg.num_shards = 64, 3 * 10**8, 64
    assert q(C.byref(cfg), 110_000_000, C.byref(sb), C.byref(wb)) == OK
    assert sb.value == (1 << 29) * 16                       # load factor 0.56 at 3e8 rows
    assert 2**30 < wb.value < 8 * 2**30
    for bad in ({"dim": 12}, {"dim": 512}, {"capacity_rows": 0}, {"capacity_rows": 2**31}, {"num_shards": 0},
                {"num_shards": 300}, {"shard_policy": 2}, {"opt": 7}):
        c2 = TableConfig()
        c2.dim, c2.capacity_rows, c2.num_shards = 16, 1000, 4
        for k, v in bad.items():
            setattr(c2, k, v)
        assert q(C.byref(c2), 100, C.byref(sb), C.byref(wb)) == ERR_INVALID_ARG, bad
    assert q(None, 100, C.byref(sb), C.byref(wb)) == ERR_INVALID_ARG
    assert q(C.byref(cfg), -1, C.byref(sb), C.byref(wb)) == ERR_INVALID_ARG
    out = C.c_void_p()
    lib.des_table_create.argtypes = [C.POINTER(TableConfig), C.POINTER(C.c_void_p)]
    assert lib.des_table_create(C.byref(cfg), C.byref(out)) == ERR_INVALID_ARG   # null buffers
    assert not out.value


def test_header_is_plain_c_and_cxx(tmp_path):
    """include/des.h compiles on its own as C99 and as C++17 (no torch, no HIP types in the signatures)."""
    import subprocess
    inc = os.path.join(ROOT, "include")
    c = tmp_path / "use.c"
    c.write_text('#include "des.h"\nint main(void) { des_table_config_t c; des_optimizer_t o; (void)c; (void)o; '
                 'return (int)sizeof(des_batch_t) == 0; }\n')
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-I", inc, str(c)])
    cpp = tmp_path / "use.cpp"
    cpp.write_text(c.read_text())
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(cpp)])
