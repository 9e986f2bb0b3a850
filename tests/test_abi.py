"""The C-ABI library loads and exports every symbol include/opevo.h declares (no GPU)."""
import ctypes
import os
import re

import paper_2006_05664_amd as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "opevo.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(opevo_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    names = _declared()
    assert len(names) >= 45
    lib = ctypes.CDLL(P.binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), "library does not export " + n
        assert callable(getattr(P, n, None)), "binding lacks " + n
    assert sorted(P.binding.EXPORTED) == names


def test_oracle_header_matches_the_oracle_library():
    """include/oracle_tensor.h: every entry point it declares is exported by the oracle's own library, and its
    prototypes agree with the definitions (the C file compiled with the header force-included)."""
    import subprocess
    from oracle import tensor as T
    header = os.path.join(ROOT, "include", "oracle_tensor.h")
    text = re.sub(r"/\*.*?\*/", "", open(header).read(), flags=re.S)
    names = sorted(set(re.findall(r"\b(oracle_[a-z0-9_]+)\s*\(", text)))
    assert names == ["oracle_bmm", "oracle_conv2d", "oracle_conv_out_extent", "oracle_matmul", "oracle_matmul_entries",
                     "oracle_matmul_rows", "oracle_num_threads", "oracle_set_threads"]
    lib = ctypes.CDLL(T.build())
    for n in names:
        assert hasattr(lib, n), "oracle library does not export " + n
    subprocess.run(["gcc", "-fsyntax-only", "-fopenmp", "-Wall", "-Werror", "-include", header,
                    os.path.join(ROOT, "oracle", "tensor_oracle.c")], check=True)
    # the product's header and sources never mention the oracle's
    assert "oracle_tensor.h" not in open(os.path.join(ROOT, "include", "opevo.h")).read()


def test_status_names_and_error_text():
    assert P.opevo_status_name(0) == "OK" and P.opevo_status_name(-3) == "E_INVALID"
    try:
        P.opevo_op_create(99, (1, 1, 1), P.OPEVO_BF16)
    except P.OpevoError as e:
        assert e.status == P.OPEVO_E_ARG and "kind" in e.message
    else:
        raise AssertionError("bad operator kind accepted")
    assert "opevo" in P.opevo_version()


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout.strip() == ""
