"""The C-ABI library loads and exports every function include/signmuon.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "signmuon.h")
LIB = os.path.join(ROOT, "paper_2605_16311_amd", "libsignmuon.so")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(signmuon_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_five_path_calls():
    names = declared_functions()
    for n in ("signmuon_momentum", "signmuon_polar_ns", "signmuon_sign_pack",
              "signmuon_majority_vote", "signmuon_step"):
        assert n in names


def test_library_exports_every_declared_symbol():
    if not os.path.exists(LIB):
        pytest.fail(f"{LIB} missing: run __graft_entry__.build() first")
    import torch  # noqa: F401  (loads the HIP runtime the library links against)
    lib = ctypes.CDLL(LIB)
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_binding_mirrors_the_abi_and_status_text():
    from paper_2605_16311_amd import binding as B
    assert set(B.EXPORTS) == set(declared_functions())
    for n in ("signmuon_momentum", "signmuon_polar_ns", "signmuon_sign_pack",
              "signmuon_majority_vote", "signmuon_step"):
        assert callable(getattr(B, n))
    assert B._lib.signmuon_strerror(0) == b"ok"
    assert B._lib.signmuon_strerror(-1) == b"invalid argument"
    assert ctypes.sizeof(B.StepArgs) == 144  # sizeof(signmuon_step_args) under the LP64 C ABI


def test_no_gpu_means_loud_failure():
    import torch
    from paper_2605_16311_amd import binding as B
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(B.SignMuonError):
        B.Context()


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2605_16311_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src, f
