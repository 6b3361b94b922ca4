"""Host-only checks of the C-ABI library: it loads, exports what the header declares, and its
pure-host entry points behave.  No kernel is launched."""
import os
import re

import numpy as np
import pytest

import gen
import paper_2502_00937_amd as V
from paper_2502_00937_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "vitenc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(vit_[a-z_]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = V.load_library()
    names = declared_symbols()
    assert {"vit_encoder_create", "vit_encode_packed", "vit_encoder_destroy", "vit_encoder_query",
            "vit_weight_count", "vit_last_error", "vit_profile_enable", "vit_profile_read",
            "vit_mfma_ceiling"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_mfma_ceiling_rejects_bad_arguments_before_touching_a_device():
    import ctypes as C

    lib = V.load_library()
    out = C.c_double(-1.0)
    assert lib.vit_mfma_ceiling(0, 0.1, 1, None) == -1      # VIT_EINVAL: NULL result pointer
    assert lib.vit_mfma_ceiling(0, 0.0, 1, C.byref(out)) == -1
    assert lib.vit_mfma_ceiling(0, 5.0, 0, C.byref(out)) == -1
    assert out.value == -1.0


def test_preprocess_rejects_bad_arguments_before_touching_a_device():
    import ctypes as C

    lib = V.load_library()
    m, sd = (C.c_float * 3)(0.5, 0.5, 0.5), (C.c_float * 3)(0.2, 0.2, 0.2)
    fake = C.c_void_p(4096)  # never dereferenced: every call below is refused on the host
    ok = dict(h=8, w=8, c=3, s=4, r=1, k=1)

    def call(img=fake, out=fake, mean=m, std=sd, cap=1 << 20, **kw):
        a = dict(ok, **kw)
        return lib.vit_preprocess_tiles(img, a["h"], a["w"], a["c"], a["s"], a["r"], a["k"], 0, mean, std, out, cap, None)

    assert call(img=None) == -1 and call(out=None) == -1 and call(mean=None) == -1 and call(std=None) == -1
    assert call(h=0) == -1 and call(c=5) == -1 and call(s=0) == -1 and call(r=0) == -1 and call(r=300, k=300) == -1
    assert call(std=(C.c_float * 3)(0.2, 0.0, 0.2)) == -1
    assert call(cap=4 * 3 * 4 * 4 - 1) == -3                 # VIT_ECAPACITY, nothing launched
    assert b"out_pixels holds" in lib.vit_last_error()


def test_header_is_valid_c99_and_cxx_and_links_from_plain_c(tmp_path):
    """The boundary is a C ABI: the header must compile as C and as C++, and a plain C program linked against
    the library must be able to call the host-only entry points."""
    import shutil
    import subprocess

    if not shutil.which("gcc") or not shutil.which("g++"):
        pytest.skip("no host compiler")
    inc = os.path.join(ROOT, "include")
    src = tmp_path / "use.c"
    src.write_text(
        '#include "vitenc.h"\n#include <stdio.h>\n'
        "int main(void) {\n"
        "  vit_config_t c = {56, 14, 3, 128, 2, 256, 2, 1, 1, 1, 1e-6f, 2, {192, 160}, VIT_DTYPE_BF16, 2};\n"
        "  size_t n = vit_weight_count(&c);\n"
        "  c.heads = 3;\n"
        '  printf("%zu %zu %s\\n", n, vit_weight_count(&c), vit_last_error());\n'
        "  return vit_encoder_create(&c, 0, 0, 0, 0) == VIT_EINVAL ? 0 : 1;\n"
        "}\n")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only", f"-I{inc}", str(src)],
                   check=True)
    cxx = tmp_path / "use.cpp"
    cxx.write_text('#include "vitenc.h"\nint main() { return vit_weight_count(nullptr) == 0 ? 0 : 1; }\n')
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", f"-I{inc}", str(cxx)], check=True)
    exe = tmp_path / "use"
    libdir = os.path.dirname(V.lib_path())
    subprocess.run(["gcc", "-std=c99", f"-I{inc}", str(src), "-o", str(exe), f"-L{libdir}", "-lvitenc",
                    f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    cfg = dict(gen.get_config("test_small_bf16"), token_merge=2)
    assert int(out[0]) == gen.weight_count(cfg) and int(out[1]) == 0


def test_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "vitenc.h")).read()
    body = text[text.index("typedef struct {"):text.index("} vit_config_t;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(?:int32_t|float)\s+([a-z_]+)(?:\[\d\])?;", body)
    assert fields == [f[0] for f in B.vit_config_t._fields_]


def test_weight_count_matches_generator_for_all_presets():
    for name in gen.CONFIGS:
        cfg = gen.get_config(name)
        assert V.vit_weight_count(cfg) == gen.weight_count(cfg), name


def test_weight_count_rejects_bad_configs():
    base = gen.get_config("test_small_bf16")
    for key, val in [("heads", 3), ("hidden", 0), ("patch_size", 0), ("proj_layers", 3), ("mlp", 7),
                     ("hidden", 20), ("has_cls", 2), ("layers_local", -1), ("ln_eps", float("nan")),
                     ("token_merge", 3), ("token_merge", -1), ("token_merge", 9),  # 56/14 = 4 is no multiple of 3
                     # sizes whose derived counts would leave 32 bits
                     ("channels", 17), ("mlp", 65544), ("layers_local", 1025), ("layers_global", 1025),
                     ("image_size", 56 * 1000), ("patch_size", 257)]:
        cfg = dict(base)
        cfg[key] = val
        if key == "proj_layers":
            cfg["proj_dims"] = (8, 8)
        assert V.vit_weight_count(cfg) == 0, (key, val)


def test_token_merge_changes_the_projector_input_only():
    base = gen.get_config("test_small_bf16")            # 4 x 4 patches, D = 128, projector 128 -> 192 -> 160
    merged = dict(base, token_merge=2)
    assert V.vit_weight_count(merged) - V.vit_weight_count(base) == 192 * 3 * 128
    assert V.vit_weight_count(dict(base, token_merge=0)) == V.vit_weight_count(base)   # 0 and 1 both mean none


def test_create_rejects_null_and_bad_arguments_without_a_device():
    lib = V.load_library()
    import ctypes as C

    handle = C.c_void_p(123)
    st = lib.vit_encoder_create(None, None, 0, 0, C.byref(handle))
    assert st == B.VIT_EINVAL and handle.value is None
    assert b"NULL" in lib.vit_last_error()
    cfg = B._to_struct(gen.get_config("test_small_bf16"))
    w = np.zeros(4, dtype=np.float32)
    st = lib.vit_encoder_create(C.byref(cfg), w.ctypes.data, w.size, 0, C.byref(handle))
    assert st == B.VIT_EINVAL and b"n_weights" in lib.vit_last_error()
    assert lib.vit_encoder_query(None, 1, 1, None, None, None, None) == B.VIT_EINVAL
    assert lib.vit_encode_packed(None, None, None, 0, None, None, 0, None, None, 0, None) == B.VIT_EINVAL
    assert lib.vit_encode_packed_graph(None, None, None, 0, None, None, 0, None, None, 0, None) == B.VIT_EINVAL
    lib.vit_encoder_destroy(None)  # NULL-safe


def test_binding_refuses_pixels_that_do_not_match_the_tile_offsets():
    """The C ABI has no pixel capacity argument; the binding checks the tensor's shape against the config and
    against tile_offsets[-1] before anything is launched."""
    cfg = gen.get_config("test_small_bf16")
    S, Cn = cfg["image_size"], cfg["channels"]
    B.check_pixels(cfg, (3, Cn, S, S), [0, 1, 3])
    for shape, to in [((3, Cn, S, S), [0, 1, 4]),          # more tiles announced than the tensor holds
                      ((3, Cn, S, S), [0, 1, 2]),          # fewer
                      ((3, Cn, S + 1, S), [0, 1, 3]),      # wrong tile size
                      ((3, Cn + 1, S, S), [0, 1, 3]),      # wrong channel count
                      ((3 * Cn * S * S,), [0, 1, 3]),      # flat
                      ((3, Cn, S, S), [])]:
        with pytest.raises(V.VitError) as e:
            B.check_pixels(cfg, shape, to)
        assert e.value.status == B.VIT_EINVAL


def test_no_cpu_fallback():
    import torch

    if torch.cuda.is_available():
        pytest.skip("GPU present")
    cfg = gen.get_config("test_small_bf16")
    with pytest.raises(RuntimeError):
        V.VitEncoder(cfg, gen.make_weights(cfg))


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2502_00937_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), os.path.join(dirpath, f)


def test_handoff_table_logic_without_a_device():
    """Everything the hand-off decides before it touches HIP: unknown / duplicate requests, missing
    images, NULL arguments (publish itself needs a device for its event)."""
    h = V.TokenHandoff(0)
    h.expect(7, 3)
    with pytest.raises(V.VitError) as e:
        h.expect(7, 1)
    assert e.value.status == -1 and "already known" in str(e.value)
    with pytest.raises(V.VitError):
        h.expect(8, 0)
    with pytest.raises(V.VitError) as e:
        h.expect(8, 65537)                  # more images than a request may announce
    assert e.value.status == -1
    h.expect(8, 65536)
    h.release(8)
    assert h.complete(7) == (False, 0)
    assert h.complete(99) == (False, 0)
    with pytest.raises(V.VitError) as e:
        h.pull(7, 4096, 1 << 20)
    assert e.value.status == -5 and "0 of 3 images" in str(e.value)  # VIT_ENOTREADY
    with pytest.raises(V.VitError) as e:
        h.pull(99, 4096, 1 << 20)
    assert e.value.status == -1
    with pytest.raises(V.VitError):
        h.publish(99, 0, 4096, 16)          # unknown request
    with pytest.raises(V.VitError):
        h.publish(7, 3, 4096, 16)           # image index out of range
    with pytest.raises(V.VitError):
        h.publish(7, 0, 0, 16)              # NULL tokens
    h.release(7)
    with pytest.raises(V.VitError):
        h.release(7)
    h.close()
