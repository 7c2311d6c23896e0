"""Host-side replay of the similarity kernel's key-row copies: for a range of candidate counts and column
splits no copy names a row outside [0, n), and every copy that is read fetches exactly its tile's rows.
The row arithmetic is the kernel's own (csrc/gram_index.h, compiled here for the CPU).  CPU only."""
import os
import subprocess

import pytest


@pytest.fixture(scope="module")
def checker(repo_root, tmp_path_factory):
    exe = tmp_path_factory.mktemp("bounds") / "gram_bounds_check"
    subprocess.run(["g++", "-O1", "-Wall", "-Werror", "-I", os.path.join(repo_root, "paper_2505_24133_amd", "csrc"),
                    "-o", str(exe), os.path.join(repo_root, "tests", "gram_bounds_check.cpp")], check=True)
    return str(exe)


def test_no_key_copy_leaves_the_candidate_rows(checker):
    # n = N - alpha for the shapes of the GPU suite that end in a partly filled tile (N = 65, 150, 1000 with
    # alpha = 8), single-tile heads, the benchmark shapes, the largest supported cache and every n below 300
    sizes = sorted(set(list(range(1, 300)) + [992, 1144, 2168, 4216, 8312, 32760, 32767]))
    for n in sizes:
        for parts in (1, 2, 3, 5, 8, 9, 16):
            r = subprocess.run([checker, str(n), str(parts)], capture_output=True, text=True)
            assert r.returncode == 0 and r.stdout.startswith("ok "), f"n={n} parts={parts}: {r.stdout}{r.stderr}"
