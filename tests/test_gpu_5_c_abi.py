"""The C ABI used from C: tests/c_abi/abi_consumer.c includes include/slicemoe.h, links the library and the C oracle, and
needs neither Python nor PyTorch.  __graft_entry__.build() compiles it; these tests run it."""
import os
import subprocess

import pytest

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "abi_consumer")


def run(*args):
    if not os.path.exists(EXE):   # built by __graft_entry__.build(); here only if nothing is built yet
        import __graft_entry__
        from paper_2510_04286_amd import binding
        import oracle
        binding.lib()
        oracle.lib()
        __graft_entry__.build_c_abi_consumer()
    r = subprocess.run([EXE, *args], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    return r


def test_c_consumer_links_and_queries_answer():
    """No GPU call: size queries, the workspace layout, and the error codes for an invalid config and null pointers."""
    r = run("--link")
    assert r.returncode == 0, r.stderr
    assert "linked" in r.stdout


@pytest.mark.gpu
def test_c_consumer_forward_matches_the_c_oracle():
    """Whole layer from C on the matrix-core path (bf16, 256 tokens, 8 slices, 16 experts): routing and dispatch tables
    against the oracle bit for bit, output within 2e-2 of RMS(h'), two runs identical, a short workspace refused."""
    r = run()
    assert r.returncode == 0, r.stdout + r.stderr
    assert "dispatch bit-exact" in r.stdout
