"""CPU check of the Python sources that only run on the GPU machine (bench.py, the binding, the entry points): every
global name a function loads is defined at module level or is a builtin.  A typo or a helper that went missing in
an edit otherwise shows up only as a NameError in the middle of a GPU run."""
import builtins
import dis
import os
import types

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FILES = ["bench.py", "__graft_entry__.py", "paper_2502_20330_amd/binding.py", "paper_2502_20330_amd/build.py",
         "paper_2502_20330_amd/workloads.py", "oracle/__init__.py", "tests/gpu_util.py"]


def _code_objects(code):
    yield code
    for c in code.co_consts:
        if isinstance(c, types.CodeType):
            yield from _code_objects(c)


@pytest.mark.parametrize("rel", FILES)
def test_every_global_name_is_defined(rel):
    path = os.path.join(ROOT, rel)
    module = compile(open(path).read(), path, "exec")
    defined = set(dir(builtins)) | {"__file__", "__name__", "__doc__", "__builtins__", "__spec__", "__package__"}
    defined |= {"__annotations__", "__qualname__", "__module__"}              # what a class body finds in its own scope
    loads = []
    for code in _code_objects(module):
        ins_list = list(dis.get_instructions(code))
        own = {i.argval for i in ins_list if i.opname == "STORE_NAME"}         # module level, or a class body's own names
        for ins in ins_list:
            if ins.opname == "STORE_GLOBAL" or (code is module and ins.opname in ("STORE_NAME", "IMPORT_NAME", "IMPORT_FROM")):
                defined.add(ins.argval.split(".")[0])
            elif ins.opname == "LOAD_GLOBAL" or (ins.opname == "LOAD_NAME" and ins.argval not in own):
                loads.append((ins.argval, code.co_name, ins.starts_line))
    # `from x import *` would hide names; none of these files uses it
    missing = sorted({(n, fn) for n, fn, _ in loads if n not in defined})
    assert not missing, f"{rel}: names loaded but never defined: {missing}"


def test_the_check_sees_a_missing_helper():
    src = "def f():\n    def g():\n        return helper(1)\n    return g()\n"
    module = compile(src, "<planted>", "exec")
    names = {ins.argval for code in _code_objects(module) for ins in dis.get_instructions(code) if ins.opname == "LOAD_GLOBAL"}
    assert "helper" in names
