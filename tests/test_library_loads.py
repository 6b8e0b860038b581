"""The C-ABI library loads and exports every function include/ann.h declares (no GPU needed)."""
import os
import re

from paper_2305_04359_amd import binding as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ann.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ann_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert "ann_build" in names and "ann_search" in names and len(names) >= 10
    lib = A.lib()
    for n in names:
        assert hasattr(lib, n), f"{n} is declared in ann.h but not exported"
    assert sorted(A.EXPORTS) == names


def test_struct_layouts_match_header():
    # field order of the ctypes mirrors follows the header text
    text = open(os.path.join(ROOT, "include", "ann.h")).read()
    def struct_body(name):
        head, _ = text.split("} " + name + ";")
        return head[head.rindex("typedef struct {") + len("typedef struct {"):]

    body = struct_body("ann_build_opts")
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = re.findall(r"(\w+)\s*;", body)
    assert fields == [f for f, _ in A.BuildOpts._fields_]
    body = struct_body("ann_hnsw_opts")
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    assert re.findall(r"(\w+)\s*;", body) == [f for f, _ in A.HnswOpts._fields_]
    body = struct_body("ann_stats")
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = [x.strip() for part in re.findall(r"(?:uint64_t|double)\s+([^;]+);", body) for x in part.split(",")]
    assert fields == [f for f, _ in A.Stats._fields_]


def test_last_error_is_callable_without_gpu():
    assert A.lib().ann_last_error() is not None
