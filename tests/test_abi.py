"""The C-ABI library loads and exports every symbol the header declares.
No compute call is made here (no GPU needed)."""
import ctypes
import os
import re

from paper_2412_18052_amd import gaf as libgaf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names.update(re.findall(r"\b(gaf_[a-z0-9_]+)\s*\(", text))
    return names


def test_header_symbols_exported():
    names = declared_symbols()
    assert {"gaf_create", "gaf_destroy", "gaf_strerror", "gaf_aggregate", "gaf_step",
            "gaf_pairwise"} <= names
    lib = libgaf.load()
    for n in sorted(names):
        assert hasattr(lib, n), "libgaf.so does not export %s" % n
    assert set(libgaf.SYMBOLS) == names


def test_strerror_is_static_text():
    assert libgaf.gaf_strerror(libgaf.GAF_OK) == "ok"
    for code in range(1, 7):
        assert libgaf.gaf_strerror(code) not in ("", "unknown status")
    assert libgaf.gaf_strerror(99) == "unknown status"


def test_null_context_is_rejected_without_a_gpu():
    lib = libgaf.load()
    assert lib.gaf_destroy(None) == libgaf.GAF_EINVAL
    assert lib.gaf_create(None, 0, 16, 1) == libgaf.GAF_EINVAL


def test_product_path_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2412_18052_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle", text, flags=re.M), fn
                assert "gaf_oracle" not in text and "oracle/" not in text, fn


def test_header_is_plain_c99():
    """include/gaf.h is the C ABI: it must compile as C, alone."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    src = "#include \"gaf.h\"\nint main(void) { return (int)GAF_OK + (int)sizeof(gaf_launch_time) * 0; }\n"
    r = subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-I",
                        os.path.join(ROOT, "include"), "-x", "c", "-"], input=src.encode(), capture_output=True)
    assert r.returncode == 0, r.stderr.decode()


def test_only_the_c_abi_is_exported():
    """Built with hidden visibility: the functions in the dynamic symbol table are the gaf_ entry
    points and nothing else (no host-side kernel stubs, no helpers)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", libgaf.LIB_PATH], capture_output=True, text=True).stdout
    funcs = {l.split()[-1] for l in out.splitlines() if len(l.split()) == 3 and l.split()[1] in "Tt"}
    assert funcs == declared_symbols(), sorted(funcs ^ declared_symbols())[:5]


def test_stale_library_is_rebuilt(tmp_path, monkeypatch):
    """load() goes through the build step's freshness check."""
    from paper_2412_18052_amd import build as hip_build
    calls = []
    monkeypatch.setattr(hip_build, "build", lambda force=True, verbose=False: calls.append(force) or hip_build.LIB)
    monkeypatch.setattr(libgaf, "_lib", None)
    libgaf.load()
    assert calls == [False]
