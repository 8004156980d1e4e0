"""Builds of oracle/jfa_oracle.c other than the committed one (a planted mistake, a sanitizer build) and the means
to run the oracle's pins against them.  CPU only; nothing here touches the HIP library."""
import importlib.util
import inspect
import os
import subprocess

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
ORACLE_DIR = os.path.join(ROOT, "oracle")
ORACLE_SRC = os.path.join(ORACLE_DIR, "jfa_oracle.c")
_count = 0


def compile_oracle(src_path, lib_path, extra_flags=()):
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", *extra_flags, "-o", lib_path, src_path, "-lm"]
    subprocess.run(cmd, check=True, capture_output=True)
    return lib_path


def oracle_module_for(lib_path):
    """A private copy of the `oracle` package module bound to another shared library."""
    global _count
    _count += 1
    spec = importlib.util.spec_from_file_location(f"oracle_variant_{_count}", os.path.join(ORACLE_DIR, "__init__.py"))
    m = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(m)
    m._LIB = lib_path
    m._lib = None
    m.build = lambda force=False: lib_path
    return m


def pin_calls(module, only=None):
    """Every (name, callable) of `module`'s tests that take the `oracle` fixture, parametrisations expanded;
    each callable takes the oracle module to check."""
    calls = []
    for name, fn in sorted(vars(module).items()):
        if not name.startswith("test_") or not callable(fn):
            continue
        params = list(inspect.signature(fn).parameters)
        if "oracle" not in params or (only and not any(name.startswith(o) for o in only)):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, lambda orc, fn=fn: fn(orc)))
            continue
        assert len(marks) == 1, name
        argnames = [a.strip() for a in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            values = values if isinstance(values, (tuple, list)) else (values,)
            kw = dict(zip(argnames, values))
            calls.append((f"{name}[{values}]", lambda orc, fn=fn, kw=kw: fn(orc, **kw)))
    return calls


if __name__ == "__main__":
    # python oracle_variants.py <library> <test name prefix> ...: run the named pins against that library (used with
    # a sanitizer build, whose runtime has to be preloaded into the interpreter, hence a process of its own)
    import sys
    sys.path.insert(0, ROOT)
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    import test_oracle_pins as pins
    orc = oracle_module_for(sys.argv[1])
    calls = pin_calls(pins, only=sys.argv[2:])
    assert calls, "no pin selected"
    for name, call in calls:
        call(orc)
        print("ok", name, flush=True)
    print(f"PINS PASSED {len(calls)}", flush=True)
