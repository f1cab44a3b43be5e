"""The C-ABI library loads without a GPU and exports every function include/helios.h declares;
host-visible argument errors are returned without touching a device."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "helios.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(helios_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2310_00837_amd import helios
    names = _declared()
    assert len(names) >= 18 and "helios_prepare_batch" in names and "helios_csr_load" in names
    lib = ctypes.CDLL(helios.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in helios.h but not exported"
    assert sorted(helios.EXPORTS) == names            # the binding knows the same list


def test_host_side_argument_errors_need_no_device():
    from paper_2310_00837_amd import helios
    lib = helios._lib
    assert lib.helios_sync(None) == helios.EINVAL
    assert lib.helios_destroy(None) == helios.EINVAL
    assert lib.helios_csr_load(None, 1, 1, None, None) == helios.EINVAL
    assert lib.helios_create(None, 0, None) == helios.EINVAL
    assert lib.helios_last_error(None) == b"no context"
    assert lib.helios_host_alloc(0) is None
    assert lib.helios_host_free(None) == helios.OK
    # plans and gangs: NULL handles and NULL member lists
    assert lib.helios_plan_launch(None, None, 0) == helios.EINVAL
    assert lib.helios_plan_wait(None) == helios.EINVAL
    assert lib.helios_plan_destroy(None) == helios.EINVAL
    out = ctypes.c_void_p()
    assert lib.helios_gang_create(None, 2, 8, None, 1, None, ctypes.byref(out)) == helios.EINVAL and not out.value
    none_ctx = (ctypes.c_void_p * 2)(None, None)
    assert lib.helios_gang_create(none_ctx, 2, 8, None, 1, None, ctypes.byref(out)) == helios.EINVAL
    assert lib.helios_gang_launch(None, None, None) == helios.EINVAL
    assert lib.helios_gang_wait(None, None) == helios.EINVAL
    assert lib.helios_gang_make_blocks(None, 0, None) == helios.EINVAL
    assert lib.helios_gang_destroy(None) == helios.EINVAL
    assert helios.MAX_GANG == 4


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2310_00837_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|helios_oracle|liboracle", src, flags=re.M), \
                    f"{f} reaches into the oracle"
