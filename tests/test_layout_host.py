"""Host-side check of the packed storage index functions (compiled for the CPU with g++):
they must be bijections onto the packed buffers, and lane l of a block must find its eight
values contiguous."""
import os
import subprocess
import tempfile

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

SRC = r'''
#include <cstdio>
#include <cstdlib>
#include <cstdint>
#define LORA_HD inline
#include "lora_layout.h"
int main(int argc, char** argv) {
  int which = atoi(argv[1]), h = atoi(argv[2]), r = atoi(argv[3]);
  if (which == 0) { for (int c = 0; c < h; ++c) for (int j = 0; j < r; ++j) printf("%lld\n", (long long)lora::packA_index(c, j, r)); }
  else { for (int j = 0; j < r; ++j) for (int d = 0; d < h; ++d) printf("%lld\n", (long long)lora::packB_index(j, d, r)); }
  return 0;
}
'''


@pytest.fixture(scope="module")
def exe():
    d = tempfile.mkdtemp()
    src = os.path.join(d, "layout_probe.cpp")
    open(src, "w").write(SRC)
    out = os.path.join(d, "layout_probe")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-I",
                           os.path.join(ROOT, "paper_2604_07173_amd", "csrc"), src, "-o", out])
    return out


def indices(exe, which, h, r):
    txt = subprocess.check_output([exe, str(which), str(h), str(r)]).decode()
    return np.array([int(t) for t in txt.split()], dtype=np.int64)


@pytest.mark.parametrize("r", [8, 16, 32, 64])
def test_packA_is_a_bijection_with_contiguous_k_runs(exe, r):
    h = 128
    ix = indices(exe, 0, h, r).reshape(h, r)
    assert sorted(ix.ravel().tolist()) == list(range(h * r))
    # eight consecutive K values of one rank index are contiguous and 16-byte aligned
    for c0 in range(0, h, 8):
        for j in range(r):
            run = ix[c0:c0 + 8, j]
            assert run[0] % 8 == 0 and np.array_equal(run, run[0] + np.arange(8))
    # one K block (32 deep, 64 for rank 8) of 16 rank indices (or all 8) is one contiguous 1 KiB
    depth = 64 if r == 8 else 32
    span = depth * min(r, 16)
    blk = ix[0:depth, 0:min(r, 16)]
    assert span == 512 and blk.min() == 0 and blk.max() == span - 1


@pytest.mark.parametrize("r", [8, 16, 32, 64])
def test_packB_is_a_bijection_and_groups_eight_columns_per_lane(exe, r):
    h = 256
    ix = indices(exe, 1, h, r).reshape(r, h)
    assert sorted(ix.ravel().tolist()) == list(range(h * r))
    run_len = 8 if r >= 32 else 4        # K values one lane holds contiguously
    for j0 in range(0, r, run_len):
        for d in range(h):
            run = ix[j0:j0 + run_len, d]
            assert run[0] % run_len == 0 and np.array_equal(run, run[0] + np.arange(run_len))
    # a 128-column chunk occupies one contiguous span of 128*r values
    assert ix[:, :128].min() == 0 and ix[:, :128].max() == 128 * r - 1
    # columns 8n .. 8n+7 belong to MFMA column slot n of sub-blocks 0..7
    if r >= 32:
        per_blk = 128 * r // 8
        for d in range(128):
            assert ix[0, d] // per_blk == d % 8
    else:
        # rank <= 16: sub-blocks come in pairs; a lane's operands of sub-blocks 2q, 2q+1 are
        # adjacent (one 16-byte load)
        per_pair = 128 * r // 4
        for d in range(128):
            assert ix[0, d] // per_pair == (d % 8) // 2
            assert (ix[0, d] // 4) % 2 == d % 2
        assert ix[0, 1] == ix[0, 0] + 4
