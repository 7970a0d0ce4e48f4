"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol,
and its host-side integer helper is exact.  No kernel is launched."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _lib():
    from paper_2505_04021_amd import build
    if not os.path.exists(build.LIB):
        build.build()
    return ctypes.CDLL(build.LIB)


def declared_in(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    text = text[text.index("extern \"C\""):]
    return set(re.findall(r"\b([a-z_0-9]+)\s*\(", text)) - {"defined"}


def declared_symbols():
    """The serving boundary (prism_kv.h) and the measurement / test hooks (prism_kv_tuning.h)."""
    return sorted(declared_in("prism_kv.h") | declared_in("prism_kv_tuning.h"))


def test_serving_header_holds_no_knobs():
    serving = declared_in("prism_kv.h")
    assert not [n for n in serving if n.startswith(("pkv_set_", "pkv_debug_", "pkv_tune", "pkv_timing", "pkv_get_xcd"))
                and n != "pkv_set_stream" and n != "pkv_set_layer"]
    assert {"pool_create", "model_register", "balloon_resize", "decode_attention"} <= serving


def test_every_declared_symbol_is_exported():
    lib = _lib()
    names = declared_symbols()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in prism_kv.h but not exported"


def test_nothing_else_is_exported():
    """The dynamic symbol table holds the declared entry points and no helper of the library's own."""
    import subprocess
    _lib()
    from paper_2505_04021_amd import build
    out = subprocess.run(["nm", "-D", "--defined-only", build.LIB], capture_output=True, text=True, check=True).stdout
    exported = sorted(line.split()[2] for line in out.splitlines() if len(line.split()) == 3 and line.split()[1] == "T")
    assert exported == declared_symbols()


def test_binding_covers_the_header():
    from paper_2505_04021_amd import binding
    assert sorted(binding.EXPORTS) == declared_symbols()


def test_fastdiv_is_exact():
    import random
    lib = _lib()
    f = lib.pkv_debug_fastdiv
    f.restype = ctypes.c_uint32
    f.argtypes = [ctypes.c_uint32, ctypes.c_uint32]
    rnd = random.Random(0)
    for d in list(range(1, 130)) + [255, 256, 257, 1000, 2048, 65535, 65536, 2**31 - 1, 2**31, 2**32 - 1]:
        for n in [0, 1, d - 1, d, d + 1, 2 * d - 1, 2 * d, 2**31 - 1, 2**31, 2**32 - 1] + \
                 [rnd.randrange(2**32) for _ in range(40)]:
            if 0 <= n < 2**32:
                assert f(n, d) == n // d, (n, d)


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2505_04021_amd")
    for root, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(root, fn)).read()
                assert "oracle" not in text.lower().replace("# no oracle", ""), fn
