"""The C-ABI library loads and exports every symbol include/hero.h declares; argument
errors are reported before any launch (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols(headers=("hero.h", "hero_debug.h")):
    names = set()
    for h in headers:
        text = open(os.path.join(ROOT, "include", h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(hero_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


@pytest.fixture(scope="module")
def lib():
    import paper_2310_17723_amd as pkg
    return pkg.load()


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2310_17723_amd import binding
    names = declared_symbols()
    assert {"hero_ln_quant", "hero_int8_gemm", "hero_int8_attn", "hero_layer_fwd"} <= set(names)
    for n in names:
        assert hasattr(lib.lib, n), f"libhero.so does not export {n}"
        assert n in binding.SYMBOLS, f"binding does not declare {n}"
    assert lib.build_arch() == "gfx950"


def test_probe_library_exports_what_its_header_declares():
    """The bench-side instruments (include/hero_probe.h) live in a library of their own; libhero does not carry them."""
    import ctypes
    from paper_2310_17723_amd import probe
    names = declared_symbols(("hero_probe.h",))
    assert set(names) == set(probe.SYMBOLS)
    plib = ctypes.CDLL(probe.LIB_PATH)
    import paper_2310_17723_amd as pkg
    for n in names:
        assert hasattr(plib, n), f"libhero_probe.so does not export {n}"
        assert not hasattr(pkg.load().lib, n), f"libhero.so still exports the bench instrument {n}"


def test_argument_errors_come_before_any_launch(lib):
    L = lib.lib
    z = C.c_float(0.0)
    # NULL pointers / bad shapes: status codes, no GPU touched
    assert L.hero_ln_quant(None, 0, None, None, 0, None, None, None, z, 4, 32, None, None, None, 0, None) == 1
    assert L.hero_ln_quant(None, 0, None, None, 0, None, None, None, z, 4, 33, None, None, None, 0, None) == 4
    assert L.hero_ln_quant(None, 0, None, None, 0, None, None, None, z, 0, 32, None, None, None, 0, None) == 0
    assert L.hero_int8_gemm(None, 64, None, None, 64, None, None, None, 0, 0, 0, None, None, 2, 64, 8, 8, 64, None) == 1
    assert L.hero_int8_gemm(None, 64, None, None, 64, None, None, None, 0, 0, 0, None, None, 2, 64, 8, 8, 60, None) == 4
    assert L.hero_int8_gemm(None, 64, None, None, 64, None, None, None, 0, 0, 0, None, None, 2, 64, -1, 8, 64, None) == 2
    assert L.hero_int8_gemm(None, 64, None, None, 64, None, None, None, 0, 0, 0, None, None, 2, 64, 0, 8, 64, None) == 0
    st = (C.c_int64 * 4)(64, 64, 64, 1)
    assert L.hero_int8_attn(None, st, None, st, None, st, 1, 1, 4, 4, 48, z, C.c_float(1.0), None, 0, 0, None, None, 0, 64, None) == 4
    assert L.hero_int8_attn(None, st, None, st, None, st, 1, 1, 4, 4, 64, z, C.c_float(1.0), None, 0, 0, None, None, 0, 64, None) == 1
    assert lib.strerror(0) == "ok" and "NULL" in lib.strerror(1)
    from paper_2310_17723_amd.binding import LayerDesc
    d = LayerDesc(0, 128, 2, 64, 256, 1e-5, 0, 31)
    n = lib.hero_layer_workspace_bytes(d, 2, 80)
    assert n >= 160 * (3 * 128 + 128 * 4 + 256) and n % 256 == 0
    assert lib.hero_layer_workspace_bytes(LayerDesc(0, 128, 2, 64, 256, 1e-5, 0, 2), 2, 80) == 0   # QKV bit clear
    assert L.hero_layer_fwd(None, None, None, None, 0, None) == 1
    # the entry point with the built-in scratch refuses a split that does not fit it (nothing is dereferenced or
    # launched on that path, so placeholder addresses do)
    fake = C.c_void_p(0x10000)
    assert lib.hero_int8_gemm_workspace_bytes(128, 4096, 16384) > (16 << 20)
    assert L.hero_int8_gemm_static(fake, 16384, None, fake, 16384, fake, None, None, 0, 0, 3, None, fake, 0, 4096,
                                   128, 4096, 16384, None) == 5
    assert L.hero_int8_gemm_static(None, 64, None, None, 64, None, None, None, 0, 0, 0, None, None, 2, 64, 8, 8, 64, None) == 1
    assert "built-in scratch" in lib.strerror(5)


def test_binding_structs_match_the_header_layout(tmp_path):
    """The three structs of hero_layer_fwd as gcc lays them out from include/hero.h against the binding's ctypes
    mirrors: size and the offset of every field (a field added to one side only would shift everything behind it)."""
    import subprocess
    from paper_2310_17723_amd import binding
    structs = {"hero_layer_desc": binding.LayerDesc, "hero_layer_weights": binding.LayerWeights, "hero_layer_io": binding.LayerIO}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "hero.h"', 'int main(void) {']
    for cname, ct in structs.items():
        lines.append(f'  printf("{cname} size %zu\\n", sizeof({cname}));')
        for f, _ in ct._fields_:
            lines.append(f'  printf("{cname} {f} %zu\\n", offsetof({cname}, {f}));')
    lines += ['  return 0;', '}']
    src, exe = tmp_path / "layout.c", tmp_path / "layout"
    src.write_text("\n".join(lines))
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = {(a, b): int(c) for a, b, c in (l.split() for l in out if l.strip())}
    for cname, ct in structs.items():
        assert seen[(cname, "size")] == C.sizeof(ct), cname
        for f, _ in ct._fields_:
            assert seen[(cname, f)] == getattr(ct, f).offset, f"{cname}.{f}"
    # and no field of the header is missing from the binding
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "hero.h")).read(), flags=re.S)
    for cname, ct in structs.items():
        body = re.search(r"typedef struct \{([^}]*)\}\s*" + cname + ";", text).group(1)
        fields = re.findall(r"\b([A-Za-z_][A-Za-z0-9_]*)\s*[;,]", body)
        assert sorted(fields) == sorted(f for f, _ in ct._fields_), cname
