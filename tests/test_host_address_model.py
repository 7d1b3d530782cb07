"""Address model: the library's sources compiled for the host and run under AddressSanitizer + UBSan.

The model (``tests/host_model``) replaces the HIP runtime header by a stand-in in which a launch is a loop over
blocks and threads and device pointers are heap pointers of exactly the tensors' sizes, so that every global
address the host and device code compute - per tile, per lane, per transfer - is checked against the extent of
its tensor.  It covers the contraction kernels with their epilogues, riders and fused column sums, the gate,
Eq.(3) and gate-gradient kernels, on layers of every alignment class with gate vectors sliced at arbitrary
offsets, rows padded to 16 bytes around ragged extents, and the store-bound kernel for ranks up to 256.  No GPU is
involved.
"""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
MODEL = os.path.join(HERE, "host_model")
CLANG = "/opt/rocm/llvm/bin/clang++"


@pytest.fixture(scope="module")
def model_binary(tmp_path_factory):
    if not os.path.exists(CLANG):
        pytest.skip("clang++ of the ROCm toolchain is not installed")
    out = str(tmp_path_factory.mktemp("address_model") / "address_model")
    cmd = [CLANG, "-std=c++17", "-O1", "-g1", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-fno-omit-frame-pointer", "-I", os.path.join(MODEL, "stub"), "-x", "c++",
           os.path.join(MODEL, "address_model.cpp"), "-o", out]
    subprocess.run(cmd, check=True, cwd=MODEL)
    return out


def _run(binary, *args):
    p = subprocess.run([binary, *args], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    tail = "\n".join(p.stdout.splitlines()[-40:])
    assert p.returncode == 0 and "address model ok" in p.stdout, tail


def test_alignment_classes(model_binary):
    # d, r, dout of every alignment class (odd, 2 mod 4, 4 mod 8, 0 mod 8) with dense last rows, riders on and
    # off, empty pending lists, boundaries with and without new gates: every 9th case of the fixed sweep
    _run(model_binary, "classes", "9")


def test_random_layers(model_binary):
    # 1-4 layers of random shape per case, gate vectors at arbitrary offsets inside one array, 0-5000 extra gates
    _run(model_binary, "random", "7", "20")


def test_padded_rows(model_binary):
    # rows padded to 16 bytes around extents that are not multiples of 8 elements: the last 16-byte chunk of every row
    # reaches into its padding; tensors end at the next multiple of 16 bytes after the last row's last element
    _run(model_binary, "padded")


def test_store_bound_kernel_for_small_ranks(model_binary):
    # outputs of 8 M and 67 M elements, so that the library takes the kernel for ranks up to 256: ranks 64, 41, 100,
    # 200 and 250 (every k-chunk variant, ranks that end inside a 16-byte piece), ragged row and column tails
    _run(model_binary, "lowrank")
