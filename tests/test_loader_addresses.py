"""The matrix kernels read their operands with unconditional, clamped 16-byte loads; an address
outside the operand is invisible to every parity test (the value is zeroed afterwards) and shows only
as a memory fault.  This test compiles the kernels' own addressing functions for the host and walks
them over every tile shape, orientation, contraction length, width, lane and K tile; likewise the
softmax-regression kernel's loads from its row-major, index-list and tiled sources."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_address_of_the_tile_loaders_lies_inside_the_operand(tmp_path):
    exe = str(tmp_path / "loader_addresses")
    src = os.path.join(ROOT, "tests", "loader_addresses.cpp")
    inc = os.path.join(ROOT, "paper_1909_07588_amd", "csrc")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-Wall", "-I" + inc, src, "-o", exe])
    r = subprocess.run([exe], capture_output=True, text=True, timeout=300)
    sys.stdout.write(r.stdout)
    assert r.returncode == 0, r.stdout[-2000:]
    lines = r.stdout.strip().splitlines()
    last = lines[-1].split()
    assert int(last[1]) > 1_000_000 and int(last[3]) == 0
    smx = [l for l in lines if l.startswith("softmax kernel: checked")][0].split()
    assert int(smx[3]) > 1_000_000 and int(smx[5]) == 0
