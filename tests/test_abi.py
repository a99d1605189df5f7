"""CPU-side checks of the boundary: the library builds/loads and exports every symbol include/kvcomp.h declares."""
import ctypes
import pathlib
import re

import pytest

ROOT = pathlib.Path(__file__).resolve().parent.parent
HEADER = ROOT / "include" / "kvcomp.h"
LIB = ROOT / "paper_2509_00579_amd" / "libkvcomp.so"


def _declared():
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(kvcomp_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    if not LIB.exists():
        from paper_2509_00579_amd import build
        build.build()
    return ctypes.CDLL(str(LIB))


def test_header_declares_the_four_hot_path_calls():
    names = _declared()
    for n in ("kvcomp_build_codebook", "kvcomp_compress_blocks", "kvcomp_append_token", "kvcomp_attn_decode"):
        assert n in names


def test_every_declared_symbol_is_exported(lib):
    for n in _declared():
        assert hasattr(lib, n), n


def test_binding_covers_every_declared_symbol():
    from paper_2509_00579_amd import binding
    assert sorted(binding.SIGNATURES) == _declared()


def test_config_validation_needs_no_gpu(lib):
    from paper_2509_00579_amd import binding
    lib.kvcomp_arena_bytes.restype = ctypes.c_size_t
    lib.kvcomp_arena_bytes.argtypes = [ctypes.POINTER(binding.Config)]
    good = binding.make_config(1, 32, 32, 4096, 1e-2, 1e-2)
    n = lib.kvcomp_arena_bytes(ctypes.byref(good))
    raw = 2 * 32 * 4096 * 128 * 2
    assert 0 < n < 1.2 * raw  # worst case (12-bit code words) stays below the fp16 size plus bookkeeping
    for bad in (binding.make_config(1, 32, 33, 4096, 1e-2, 1e-2),      # heads do not divide
                binding.make_config(1, 8, 24, 4096, 1e-2, 1e-2),       # group of 3 unsupported
                binding.make_config(1, 32, 32, 4096, 0.6, 1e-2),       # error bound above 1/2
                binding.make_config(1, 32, 32, 4096, 1e-2, 1e-4),      # more than 256 levels
                binding.make_config(0, 32, 32, 4096, 1e-2, 1e-2),
                binding.make_config(1, 32, 32, 4096, 1e-2, 1e-2, max_code_len=13)):
        assert lib.kvcomp_arena_bytes(ctypes.byref(bad)) == 0
    lib.kvcomp_baseline_workspace_bytes.restype = ctypes.c_size_t
    lib.kvcomp_baseline_workspace_bytes.argtypes = [ctypes.POINTER(binding.Config)]
    assert lib.kvcomp_baseline_workspace_bytes(ctypes.byref(good)) == 32 * 128 * 130 * 4 + 32 * 4   # 128 split partials per query head + the tickets


def test_library_codebook_matches_oracle_rules_without_a_gpu():
    # the host-side codebook builder is reachable only through a context (needs a GPU); its parity is covered by the
    # gpu tests.  Here: the product package must not import the oracle.
    import paper_2509_00579_amd.binding as b
    src = pathlib.Path(b.__file__).read_text()
    assert "oracle" not in src


def _prototypes():
    """name -> list of parameter declarations, parsed from the header."""
    text = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    text = re.sub(r"//[^\n]*", "", text)
    out = {}
    for m in re.finditer(r"\b(kvcomp_[a-z0-9_]+)\s*\(([^)]*)\)\s*;", text):
        params = [p.strip() for p in m.group(2).split(",")]
        out[m.group(1)] = [] if params in ([""], ["void"]) else params
    return out


def _kind(decl):
    """Class of a C parameter as the binding has to marshal it."""
    if "*" in decl:
        return "pointer"
    base = re.sub(r"\b(const|unsigned|signed)\b", "", decl).split()
    return {"int": "int", "float": "float", "size_t": "size_t"}[base[0]]


def test_binding_argument_lists_follow_the_header():
    from paper_2509_00579_amd import binding
    protos = _prototypes()
    assert sorted(protos) == _declared()
    kinds = {ctypes.c_int: "int", ctypes.c_float: "float", ctypes.c_size_t: "size_t"}
    for name, (_, args) in binding.SIGNATURES.items():
        want = [_kind(p) for p in protos[name]]
        got = [kinds.get(a, "pointer") for a in args]
        assert got == want, (name, protos[name])
