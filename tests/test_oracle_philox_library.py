"""The oracle's Philox4x32-10 (the generator behind the RandomLLM baseline, paper Sec. 4.1) against an
implementation that is not this repository's: the engine in the rocRAND headers that ship with ROCm, which host
code can call.  A small driver (tests/philox/rocrand_philox_driver.cpp) is compiled here and fed (seed,
subsequence, block) triples; the oracle must return the same four words for the matching (counter, key).  Together
with the three published known-answer vectors this pins every word of the counter, both key words and all four
output words, on hundreds of inputs."""
import os
import shutil
import subprocess

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    if not (os.path.exists(HIPCC) or shutil.which(HIPCC)):
        pytest.skip("hipcc not available")
    exe = str(tmp_path_factory.mktemp("philox") / "rocrand_philox_driver")
    src = os.path.join(ROOT, "tests", "philox", "rocrand_philox_driver.cpp")
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-O1", src, "-o", exe], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def library_blocks(exe, triples):
    text = "".join(f"{s} {q} {c}\n" for s, q, c in triples)
    r = subprocess.run([exe], input=text, capture_output=True, text=True, timeout=60)
    assert r.returncode == 0, r.stderr
    rows = [[int(w, 16) for w in line.split()] for line in r.stdout.splitlines()]
    assert len(rows) == len(triples)
    return np.array(rows, dtype=np.uint64)


def test_oracle_philox_matches_the_rocrand_engine(driver, ref):
    rng = np.random.default_rng(20240528)
    triples = [(0, 0, 0), (1, 0, 0), (0, 1, 0), (0, 0, 1), (2 ** 64 - 1, 2 ** 64 - 1, 2 ** 62 - 1),
               (2 ** 32, 0, 0), (0, 2 ** 32, 0), (0, 0, 2 ** 32), (2 ** 32 - 1, 2 ** 32 - 1, 2 ** 32 - 1)]
    for _ in range(400):
        width = [int(rng.integers(1, 65)) for _ in range(3)]
        s, q, c = (int(rng.integers(0, 2 ** 63, dtype=np.uint64)) >> (63 - min(w, 63)) for w in width)
        triples.append((s, q, min(c, 2 ** 62 - 1)))
    got = library_blocks(driver, triples)
    for (s, q, c), want in zip(triples, got):
        ctr = [c & 0xffffffff, c >> 32, q & 0xffffffff, q >> 32]
        key = [s & 0xffffffff, s >> 32]
        out = ref.philox4x32_10(ctr, key)
        assert [int(x) for x in out] == [int(x) for x in want], (s, q, c)


def test_the_baselines_keys_are_that_generators_word_0(driver, ref):
    """RandomLLM ranks slot i of stream s at turn t under seed k by word 0 of the block with counter
    {i, s, t low word, t high word} and key {k low word, k high word}.  In the library's terms that is seed k,
    subsequence t and block number (s << 32) | i."""
    rng = np.random.default_rng(7)
    triples, want_inputs = [], []
    for _ in range(100):
        i, s = int(rng.integers(0, 2 ** 24)), int(rng.integers(0, 2 ** 16))
        t, k = int(rng.integers(0, 2 ** 63, dtype=np.uint64)), int(rng.integers(0, 2 ** 63, dtype=np.uint64))
        block = (s << 32) | i
        triples.append((k, t, block))
        want_inputs.append(([i, s, t & 0xffffffff, t >> 32], [k & 0xffffffff, k >> 32]))
    got = library_blocks(driver, triples)
    for (ctr, key), want in zip(want_inputs, got):
        assert int(ref.philox4x32_10(ctr, key)[0]) == int(want[0])
