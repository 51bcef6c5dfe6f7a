"""The C-ABI library loads without a GPU and exports every function include/aet_sgd.h
declares.  No compute call is made here."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "aet_sgd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aet_[a-zA-Z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_named_calls():
    names = declared_functions()
    for must in ("aet_init", "aet_run_round", "aet_server_aggregate"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2112_13935_amd import build
    from paper_2112_13935_amd.binding import EXPORTS
    if build.needs_build():
        build.build(force=True)
    lib = ctypes.CDLL(build.LIB)
    names = declared_functions()
    assert names, "no declarations found"
    for name in names:
        assert hasattr(lib, name), f"{name} is declared but not exported"
    assert sorted(EXPORTS) == names, "binding and header disagree on the entry points"


def test_model_validation_runs_on_the_host():
    """aet_n_params / aet_workspace_bytes are pure host arithmetic."""
    import workloads as W
    from paper_2112_13935_amd.binding import load_library, model_desc
    lib = load_library()
    for model, want in ((W.softmax_model(784, 10), 7850), (W.mlp_model(784, 128, 10, 32), 101770),
                        (W.lenet_model(16), 44426), (W.cnn32_model(64), 1116970),
                        (W.softmax_model(3072, 10), 30730)):
        d = model_desc(model)
        assert lib.aet_n_params(ctypes.byref(d)) == want
        assert lib.aet_workspace_bytes(ctypes.byref(d), 4, 2, 10) > 4 * want * 4
    bad = model_desc(W.Model(1, 7, 7, [W.Layer(W.CONV, 2, 3, 0, 1), W.Layer(W.POOL), W.Layer(W.DENSE, 3)], 2))
    assert lib.aet_n_params(ctypes.byref(bad)) == -1          # 5x5 map cannot be pooled 2x2
    assert lib.aet_workspace_bytes(ctypes.byref(bad), 4, 1, 1) == 0
    ok = model_desc(W.softmax_model(8, 3))
    assert lib.aet_workspace_bytes(ctypes.byref(ok), 0, 1, 1) == 0
