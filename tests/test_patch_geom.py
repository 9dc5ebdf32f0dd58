"""Index arithmetic of the GPU library's input-patch convolution, built for the host (CPU only):
every tile, output pixel and filter tap must land on the input pixel the convolution's definition
names, inside the patch, and the patch must respect its closed-form size bound."""
import os
import subprocess

import pytest

import sparq_synth as S

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def checker(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("geom") / "patch_geom_check")
    subprocess.run(["g++", "-O2", "-std=c++17", "-o", exe, os.path.join(HERE, "patch_geom_check.cpp")], check=True)
    return exe


def _layer_shapes():
    seen = {}
    for layers in (S.config0(), S.config1(), S.config2(batch=4), S.config4(batch=3)):
        for l in layers:
            seen[(l.B, l.H, l.W, l.KH, l.KW, l.stride[0], l.stride[1], l.pad[0], l.pad[1])] = l.name
    return sorted(seen)


EXTRA = [(3, 7, 7, 3, 3, 1, 1, 1, 1), (64, 32, 32, 3, 3, 1, 1, 1, 1), (1, 1, 100000, 1, 1, 1, 1, 0, 0),
         (300, 1, 1, 1, 1, 1, 1, 0, 0), (7, 3, 5, 3, 3, 1, 1, 2, 2), (2, 230, 230, 3, 3, 1, 1, 1, 1),
         (5, 9, 11, 2, 4, 2, 3, 1, 2), (2, 40, 130, 3, 3, 1, 1, 0, 0), (9, 5, 4, 5, 3, 1, 1, 2, 1),
         (2, 129, 3, 3, 3, 1, 2, 1, 1), (1, 128, 128, 3, 3, 1, 1, 1, 1), (3, 16, 16, 1, 1, 1, 1, 0, 0),
         (11, 6, 6, 3, 3, 3, 3, 0, 0), (4, 12, 12, 1, 1, 2, 2, 0, 0)]


@pytest.mark.parametrize("shape", _layer_shapes() + EXTRA, ids=lambda s: "x".join(map(str, s)))
def test_patch_indexing_matches_the_convolution(checker, shape):
    r = subprocess.run([checker, *map(str, shape)], capture_output=True, text=True)
    assert r.returncode == 0 and r.stdout.startswith("ok"), r.stdout + r.stderr
