"""The package's example (an empty pool, one request admitted, a second one that finds the first
one's chunks at shifted positions) runs and reports what it should."""
import pytest
import torch

pytestmark = pytest.mark.gpu


def test_example_serves_from_what_it_admitted():
    assert torch.cuda.is_available(), "GPU tests need an MI355X; deselect with -m 'not gpu'"
    from paper_2605_05696_amd import example
    r = example.main()
    chunks, hits, admitted = r["first"]
    assert hits == 0 and admitted == chunks - 1            # the first chunk sits inside the carve-out
    chunks2, hits2, hit_tokens = r["second"]
    assert hits2 >= chunks2 - 3 and hit_tokens > 3000      # all but the chunks around the fresh head
    assert r["delta"] < 0 and r["ckv_identical"]


def test_plain_c_client_of_the_library():
    """csrc/abi_client.c, built by gcc as C99 against the public header, drives the four calls from C
    and checks their results itself (a child process: no Python object crosses the boundary)."""
    import os
    import subprocess
    from paper_2605_05696_amd import build
    if not os.path.exists(build.CLIENT):                   # built with the library; a second of gcc if it is not there
        try:
            build.build_client()
        except (OSError, subprocess.CalledProcessError) as e:
            pytest.skip(f"no C client and no way to build it here: {e}")
    r = subprocess.run([build.CLIENT], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert r.stdout.startswith("abi_client ok:"), r.stdout
