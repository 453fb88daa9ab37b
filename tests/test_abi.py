"""CPU-side checks of the boundary: the shared library loads, exports every
symbol the header declares, builds the same codebook as the oracle, and
rejects bad arguments with a status code before touching the GPU."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import workloads as W
from oracle import turboquant_oracle as o

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2504_19874_amd import _lib
    if not os.path.exists(_lib.LIB_PATH):
        from paper_2504_19874_amd import build
        build.build_library(verbose=False)
    return _lib.load()


def header_functions():
    text = open(os.path.join(ROOT, "include", "turboquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tq_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2504_19874_amd import _lib
    names = header_functions()
    assert {"tq_build_codebook", "tq_quantize_mse", "tq_quantize_prod", "tq_dequantize", "tq_score"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
        assert n in _lib.SIGNATURES, f"{n} has no ctypes signature"
    assert set(_lib.SIGNATURES) == set(names)


def test_params_struct_matches_header_layout():
    from paper_2504_19874_amd import _lib
    # int32 x2, 9 pointer-sized fields, then the split: int32 x2 and two pointers, then the flags word (padded)
    # and the pointer to the parameter images
    assert C.sizeof(_lib.TqParams) == 8 + 9 * 8 + 8 + 2 * 8 + 8 + 8
    assert _lib.TqParams.flags.offset == 104 and _lib.TqParams.images.offset == 112
    assert _lib.TqParams.Pi.offset == 8 and _lib.TqParams.workspace_bytes.offset == 72
    assert _lib.TqParams.d_hi.offset == 80 and _lib.TqParams.bits_mse_hi.offset == 84
    assert _lib.TqParams.centroids_hi.offset == 88 and _lib.TqParams.bounds_hi.offset == 96


@pytest.mark.parametrize("d,bits", [(3, 2), (8, 3), (128, 1), (128, 2), (128, 3), (128, 4), (1536, 4), (3072, 1), (200, 5)])
def test_codebook_builder_matches_oracle(lib, d, bits):
    import paper_2504_19874_amd as tq
    c, t, cost = tq.tq_build_codebook(d, bits)
    c64, t64, cost_o = o.lloyd_max_codebook(d, bits)
    assert np.max(np.abs(c - c64)) < 1e-7 / np.sqrt(d) and np.max(np.abs(t - t64)) < 1e-7 / np.sqrt(d)
    assert np.array_equal(c, c64.astype(np.float32)) and np.array_equal(t, t64.astype(np.float32))
    assert abs(cost / cost_o - 1) < 1e-8
    assert np.array_equal(c, -c[::-1])


def test_codebook_builder_rejects_bad_arguments(lib):
    buf = (C.c_float * 256)()
    assert lib.tq_build_codebook(2, 1, buf, buf, None) == 1
    assert lib.tq_build_codebook(128, 9, buf, buf, None) == 1
    assert lib.tq_build_codebook(128, 2, None, buf, None) == 1
    assert lib.tq_build_codebook(128, 0, buf, None, None) == 0 and buf[0] == 0.0
    assert lib.tq_status_string(0) == b"TQ_OK" and lib.tq_status_string(2) == b"TQ_ERR_UNSUPPORTED"


def test_entry_points_validate_before_launching(lib):
    from paper_2504_19874_amd import _lib
    c = np.zeros(4, dtype=np.float32)
    t = np.zeros(3, dtype=np.float32)
    p = _lib.TqParams()
    p.d, p.bits_mse = 100, 2  # not a multiple of 32
    p.centroids, p.bounds = c.ctypes.data, t.ctypes.data
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 100, None, None, None) == 2
    p.d = 128
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 128, None, None, None) == 1  # NULL x
    assert lib.tq_quantize_mse(C.byref(p), None, 0, -1, 128, None, None, None) == 1
    assert lib.tq_quantize_mse(C.byref(p), None, 7, 4, 128, None, None, None) == 1   # bad dtype
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 0, 128, None, None, None) == 0   # empty input is fine
    p.bits_mse = 5
    assert lib.tq_dequantize(C.byref(p), None, None, None, None, 1, None, 128, None) == 2
    p.bits_mse = 2
    assert lib.tq_dequantize(C.byref(p), None, None, None, None, 1, None, 128, None) == 1
    assert lib.tq_score(C.byref(p), None, 128, 1, 1, None, None, None, None, 10, None, 10, 0, None, None, None) == 1
    assert lib.tq_score(C.byref(p), None, 128, 1, 1, None, None, None, None, 10, None, 10, 65, None, None, None) == 2
    assert lib.tq_stage_sign_pack(100, None, 1, None, None) == 2
    assert lib.tq_workspace_bytes(C.byref(p), 1000, 10, 0) >= 1000 * 128 * 4 + 2 * 10 * 128 * 4
    assert lib.tq_derive_params(128, None, None, None, None, None, None) == 1
    # parameter images: sizes, and nothing is launched for missing matrices or dimensions that take none
    assert lib.tq_images_bytes(128) == (5 + 4) * 128 * 128 * 2 and lib.tq_images_bytes(1536) == 10 * 1536 * 1536
    assert lib.tq_images_bytes(100) == 0 and lib.tq_images_bytes(0) == 0
    assert lib.tq_build_images(None, None, None) == 1
    assert lib.tq_build_images(C.byref(p), None, None) == 1          # d = 128, no buffer and no matrices
    q = _lib.TqParams()
    q.d = 100
    assert lib.tq_build_images(C.byref(q), None, None) == 0          # no image at this dimension: a no-op
    # two instances over a channel split: what is malformed, and what the kernels do not cover
    c_hi = np.zeros(8, dtype=np.float32)
    t_hi = np.zeros(7, dtype=np.float32)
    p.d_hi, p.bits_mse_hi = 48, 3  # not a multiple of 32
    p.centroids_hi, p.bounds_hi = c_hi.ctypes.data, t_hi.ctypes.data
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 128, None, None, None) == 1
    p.d_hi = 128  # no channel left for the other instance
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 128, None, None, None) == 1
    p.d_hi, p.centroids_hi = 32, None
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 128, None, None, None) == 1
    p.centroids_hi, p.bits_mse_hi = c_hi.ctypes.data, 2  # the outlier instance must have one more bit
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 128, None, None, None) == 2
    p.bits_mse_hi, p.d, p.d_hi = 3, 256, 64  # head dimension 128 only
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 4, 256, None, None, None) == 2
    p.d, p.d_hi = 128, 64
    assert lib.tq_quantize_mse(C.byref(p), None, 0, 0, 128, None, None, None) == 0   # valid and empty
    assert lib.tq_stage_pack(C.byref(p), None, 4, None, None) == 2                   # stages know one instance


def test_rotation_helper_agrees_with_oracle_reading():
    import paper_2504_19874_amd as tq
    G = W.gaussian_matrix(96, 42)
    a = tq.rotation_from_gaussian(G).numpy()
    b = o.rotation_from_gaussian(G)
    assert np.max(np.abs(a.astype(np.float64) - b.astype(np.float64))) < 1e-6
    R = a.astype(np.float64).T @ G
    assert np.all(np.diag(R) > 0) and np.max(np.abs(np.tril(R, -1))) < 1e-5


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2504_19874_amd import _lib
    monkeypatch.setattr(_lib, "_lib", None)
    monkeypatch.setattr(_lib, "LIB_PATH", "/nonexistent/libturboquant.so")
    with pytest.raises(RuntimeError, match="no CPU or PyTorch fallback"):
        _lib.load()


def test_workload_generators_are_seeded_and_shaped():
    a = W.kv_keys_chunk(1, 0, 300, 128, 2, W.kv_outlier_channels(8, 128, 2))
    b = W.kv_keys(2, 300, 128, 2)[1]
    assert a.dtype == np.uint16 and np.array_equal(a, b)
    v = o.bf16_bits_to_f64(a)
    out = W.kv_outlier_channels(8, 128, 2)[1]
    assert v[:, out].std() > 10 and np.delete(v, out, axis=1).std() < 1.2
    c = W.mixture_centers(64, 4)
    m1 = W.mixture_chunk(0, 100, 64, 4, c)
    m2 = W.mixture_chunk(0, 50, 64, 4, c)
    assert np.allclose(np.linalg.norm(m1, axis=1), 1, atol=1e-6) and m1.dtype == np.float32
    assert W.CONFIGS["C5"].bits_mse == 1 and W.CONFIGS["C4"].bits_mse == 4


def test_split_composer_places_blocks_on_their_channels(lib):
    import paper_2504_19874_amd as tq
    from paper_2504_19874_amd import params
    d, hi = 12, [7, 2, 9]
    rng = np.random.default_rng(5)
    a = rng.standard_normal((3, 3)).astype(np.float32)
    b = rng.standard_normal((9, 9)).astype(np.float32)
    got = params.compose_split(d, hi, a, b).numpy()
    x = rng.standard_normal(d).astype(np.float32)
    hi_sorted = sorted(hi)
    lo = [c for c in range(d) if c not in hi]
    # the composed matrix applies block a to the hi channels and block b to the others, each in ascending order
    want = np.concatenate([a @ x[hi_sorted], b @ x[lo]])
    assert np.allclose(got @ x, want, atol=1e-6)
    assert np.count_nonzero(got) <= 9 + 81


def test_host_code_under_address_and_undefined_sanitizers(lib, tmp_path):
    """The library's CPU code (codebook solver, rotation builder, split composer, entropy codec, and the argument checks of
    every entry point) compiled with -fsanitize=address,undefined on the host side and driven by
    tests/host/sanitize_driver.cpp; device code objects are linked in as built, nothing touches a GPU."""
    import glob
    import shutil
    import subprocess
    from paper_2504_19874_amd import build
    if shutil.which("hipcc") is None:
        pytest.skip("no hipcc")
    objs = [f for f in glob.glob(os.path.join(build.OBJ, "*.o"))
            if os.path.basename(f) not in ("tq_api.o", "tq_codebook.o", "tq_rotation.o", "tq_entropy.o")]
    if len(objs) < len(build.SOURCES) - 4:
        build.build_library(verbose=False)
        objs = [f for f in glob.glob(os.path.join(build.OBJ, "*.o"))
                if os.path.basename(f) not in ("tq_api.o", "tq_codebook.o", "tq_rotation.o", "tq_entropy.o")]
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    host = ["hipcc", "-O1", "-g", "-std=c++17", "-x", "c++", *san, "-c"]
    made = []
    for src in (os.path.join(build.CSRC, "tq_codebook.cpp"), os.path.join(build.CSRC, "tq_rotation.cpp"),
                os.path.join(build.CSRC, "tq_entropy.cpp"),
                os.path.join(ROOT, "tests", "host", "sanitize_driver.cpp")):
        out = str(tmp_path / (os.path.basename(src) + ".o"))
        subprocess.run([*host, src, "-o", out], check=True, capture_output=True)
        made.append(out)
    api_o = str(tmp_path / "tq_api.o")
    xh = [f for s in san for f in ("-Xarch_host", s)]
    subprocess.run(["hipcc", *[f for f in build.HIP_FLAGS if f != "-O3"], "-O1", "-g", *xh, "-c",
                    os.path.join(build.CSRC, "tq_api.hip"), "-o", api_o], check=True, capture_output=True)
    exe = str(tmp_path / "sanitize_driver")
    subprocess.run(["hipcc", "--offload-arch=gfx950", *san, "-o", exe, *made, api_o, *objs], check=True,
                   capture_output=True)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "argument checks ok" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr


def test_binding_rejects_short_or_mistyped_code_tensors():
    """The library sees addresses only; the binding checks every code tensor against the call's sizes."""
    import torch
    from paper_2504_19874_amd import api

    class Shape:
        idx_words, qjl_words, scalars_per_vector = 8, 4, 1

    good = dict(idx=torch.zeros(80, dtype=torch.int32), qjl=torch.zeros(40, dtype=torch.int32),
                gamma=torch.zeros(10), norm=torch.zeros(10))
    api._check_codes(Shape, 10, **good)
    for key, bad in [("idx", torch.zeros(79, dtype=torch.int32)), ("idx", torch.zeros(80, dtype=torch.int64)),
                     ("qjl", torch.zeros(39, dtype=torch.int32)), ("gamma", torch.zeros(9)),
                     ("norm", torch.zeros(10, dtype=torch.float64))]:
        with pytest.raises(api.TurboQuantError, match=key):
            api._check_codes(Shape, 10, **{**good, key: bad})
    q = torch.zeros((8, 128))
    with pytest.raises(api.TurboQuantError, match="scores"):
        api._check_score_args(Shape, q, 2, 4, good["idx"], None, None, None, 5, torch.zeros((8, 4)), 0, None, None)
    with pytest.raises(api.TurboQuantError, match="topk_idx"):
        api._check_score_args(Shape, q, 2, 4, good["idx"], None, None, None, 5, None, 3,
                              torch.zeros(23, dtype=torch.int32), None)
    with pytest.raises(api.TurboQuantError, match="q:"):
        api._check_score_args(Shape, q[:7], 2, 4, good["idx"], None, None, None, 5, None, 3,
                              torch.zeros(24, dtype=torch.int32), None)
