"""The C-ABI library loads and exports every symbol that include/mmee.h declares.
No compute call is made here (no GPU needed); host-only entry points are exercised."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mmee.h")
LIB = os.path.join(ROOT, "paper_2604_03446_amd", "libmmee.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mmee_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_problem_statement():
    names = declared_functions()
    for required in ("mmee_space_size", "mmee_eval_batch", "mmee_search"):
        assert required in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        import __graft_entry__ as g
        g.build()
    lib = ctypes.CDLL(LIB)
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_binding_mirrors_the_header():
    import paper_2604_03446_amd as M
    for name in declared_functions():
        if name == "mmee_strerror":
            continue
        assert callable(getattr(M, name)), name
    assert ctypes.sizeof(M.Cost) == 64
    assert ctypes.sizeof(M.Mapping) == 56


def test_host_only_calls():
    import paper_2604_03446_amd as M
    from inputs import CONFIGS
    sizes = {k: M.mmee_space_size(c["workload"], c["hw"]) for k, c in CONFIGS.items()}
    assert sizes == {"tiny": 952560000, "bert": 2646000000, "prefill": 4976640000, "long": 6773760000}
    with pytest.raises(M.MmeeError) as e:
        M.mmee_space_size(dict(CONFIGS["tiny"]["workload"], d=0), CONFIGS["tiny"]["hw"])
    assert e.value.code == M.EINVAL
    # a workload whose counts would not stay exact integers in fp64 is refused, not approximated
    with pytest.raises(M.MmeeError):
        M.mmee_space_size(dict(CONFIGS["tiny"]["workload"], N=1 << 20, d=1 << 10, H=1 << 10), CONFIGS["tiny"]["hw"])
