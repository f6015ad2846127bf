"""The C-ABI library loads and exports every function include/hisa.h declares (no GPU, no compute calls)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "hisa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hisa_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_1810_00845_amd import hisa
    lib = hisa.load()
    names = declared_functions()
    assert len(names) > 60 and "hisa_rot_left_batch" in names and "hisa_conv2d" in names
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing


def test_create_rejects_bad_parameters_or_reports_no_gpu():
    """Argument checks run before any device work; with no GPU the call must fail, never fall back."""
    from paper_1810_00845_amd import hisa
    lib = hisa.load()
    prm = hisa.Params()
    prm.log_n, prm.num_q, prm.dnum, prm.special_bits = 9, 1, 1, 50   # log_n below the supported range
    prm.q_bits[0] = 50
    h = ctypes.c_void_p()
    assert lib.hisa_create(ctypes.byref(prm), None, ctypes.byref(h)) == -1 and not h.value
    prm.log_n, prm.dnum = 12, 2                                       # more digits than primes
    assert lib.hisa_create(ctypes.byref(prm), None, ctypes.byref(h)) == -1
    assert lib.hisa_create(None, None, ctypes.byref(h)) == -1
    assert lib.hisa_free(None, None) == 0
    assert lib.hisa_conv2d_apply_multi(None, None, None, ctypes.c_size_t(0), None) == -1
    assert lib.hisa_conv2d_apply(None, None, None, None) == -1
    assert lib.hisa_last_error(None) == b"no context"


def test_binding_mirrors_the_header():
    """Every HISA instruction of the header has a method of the same name (minus the prefix) on the binding."""
    from paper_1810_00845_amd import hisa
    skip = {"hisa_create", "hisa_destroy", "hisa_last_error", "hisa_free", "hisa_get_primes", "hisa_get_alpha",
            "hisa_ct_info", "hisa_pt_info", "hisa_tensor_free", "hisa_ct_device_ptr"}
    for n in declared_functions():
        if n in skip:
            continue
        assert hasattr(hisa.Context, n[len("hisa_"):]), n


def test_binding_structs_have_the_layout_of_the_header(tmp_path):
    """The ctypes structures of the binding against the C compiler's view of include/hisa.h: size of every struct that
    crosses the boundary by pointer, and the offset of the last field of each."""
    import subprocess
    from paper_1810_00845_amd import hisa
    pairs = [("hisa_params", hisa.Params, "hamming_weight"), ("hisa_op_counts", hisa.OpCounts, "limb_sq_sum"),
             ("hisa_tensor", hisa.TensorStruct, "cts"), ("hisa_conv_geom", hisa.ConvGeom, "chw_schedule"),
             ("hisa_calibration", hisa.Calibration, "reserved"), ("hisa_mac_extents", hisa.MacExtents, "w_extent")]
    src = tmp_path / "layout.c"
    body = "\n".join('    printf("%s %%zu %%zu\\n", sizeof(%s), offsetof(%s, %s));' % (c, c, c, last) for c, _, last in pairs)
    src.write_text('#include <stdio.h>\n#include <stddef.h>\n#include "hisa.h"\nint main(void) {\n%s\n    return 0;\n}\n' % body)
    exe = tmp_path / "layout"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = subprocess.check_output([str(exe)]).decode().split("\n")
    seen = {line.split()[0]: (int(line.split()[1]), int(line.split()[2])) for line in out if line.strip()}
    for cname, struct, last in pairs:
        assert seen[cname] == (ctypes.sizeof(struct), getattr(struct, last).offset), (cname, seen[cname])
