"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, its host-only routine agrees with the oracle, and device calls fail cleanly
(never fall back to a CPU path) when no GPU is there."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import chebyshev as ocheb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "dash.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2602_02016_amd import load_library
    from paper_2602_02016_amd.binding import LIB_PATH
    if not os.path.exists(LIB_PATH):
        from paper_2602_02016_amd.build import build_library
        build_library(verbose=False)
    return load_library()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dash_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = _declared_functions()
    assert {"dash_create", "dash_accumulate_factors", "dash_inverse_root", "dash_precondition", "dash_step",
            "dash_chebyshev_fit", "dash_gemm_batched", "dash_block_norms", "dash_graft_update"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in dash.h but not exported"


def test_step_args_layout_matches_header():
    # the ctypes mirror must list the header's fields in the header's order
    from paper_2602_02016_amd.binding import _StepArgs
    text = open(HEADER).read()
    body = text[text.index("typedef struct {", text.index("one optimizer step")):text.index("} dash_step_args;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.replace("typedef struct {", "").strip()
        if not decl:
            continue
        names = decl.split(",")
        first = names[0].split()[-1].lstrip("*")
        fields.append(first)
        fields += [n.strip().lstrip("*") for n in names[1:]]
    assert fields == [f[0] for f in _StepArgs._fields_]


def _struct_fields(text, typedef_name):
    end = text.index("} " + typedef_name + ";")
    body = text[text.rindex("typedef struct {", 0, end):end]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.replace("typedef struct {", "").strip()
        if not decl:
            continue
        names = decl.split(",")
        fields.append(names[0].split()[-1].lstrip("*"))
        fields += [n.strip().lstrip("*") for n in names[1:]]
    return fields


def test_model_structs_match_header():
    from paper_2602_02016_amd.binding import _LayerShape, _ModelInfo, _ModelStepArgs
    text = open(HEADER).read()
    assert _struct_fields(text, "dash_layer_shape") == [f[0] for f in _LayerShape._fields_]
    assert _struct_fields(text, "dash_model_info") == [f[0] for f in _ModelInfo._fields_]
    assert _struct_fields(text, "dash_model_step_args") == [f[0] for f in _ModelStepArgs._fields_]


@pytest.mark.parametrize("p,d,a,b,n", [(2, 8, 0.01, 1.0, 1000), (4, 16, 1e-3, 1.001, 10000), (4, 60, 1e-6, 1.000001, 10000)])
def test_host_chebyshev_fit_matches_oracle(lib, p, d, a, b, n):
    from paper_2602_02016_amd import chebyshev_fit
    c = np.array(chebyshev_fit(p, d, a, b, n))
    ref = ocheb.chebyshev_fit(p, d, a, b, n)
    assert np.allclose(c, ref, rtol=1e-12, atol=1e-12 * np.abs(ref).max())


def test_host_chebyshev_fit_rejects_bad_arguments(lib):
    out = (ctypes.c_double * 8)()
    assert lib.dash_chebyshev_fit(3, 4, 0.1, 1.0, 100, out) == 1     # p
    assert lib.dash_chebyshev_fit(2, 4, 1.0, 0.5, 100, out) == 1     # b <= a
    assert lib.dash_chebyshev_fit(2, 4, 0.0, 1.0, 100, out) == 1     # a must be > 0 for x^(-1/p)
    assert lib.dash_chebyshev_fit(2, 4, 0.1, 1.0, 3, out) == 1       # fewer points than coefficients
    assert lib.dash_chebyshev_fit(2, 4, 0.1, 1.0, 100, None) == 1


def test_workspace_size_formula(lib):
    # Newton-DB keeps five B x B fp32 buffers per block, Clenshaw three; on top of that the scaling
    # step keeps per block two B x 32 pool buffers (multi-Power-Iteration), the per-workgroup partial sums
    # of its sweeps (two buffers of 32 + 64 * B/128 floats) and a few scalars
    mat = 1024 * 1024 * 4
    extra = 32 * (2 * 1024 * 32 * 4 + 2 * (32 + 64 * 8) * 4 + 1024)
    n5 = lib.dash_workspace_bytes(32, 1024, 0, 4, 0)
    n3 = lib.dash_workspace_bytes(32, 1024, 1, 4, 0)
    assert 32 * 5 * mat <= n5 < 32 * 5 * mat + extra + (1 << 16)
    assert 32 * 3 * mat <= n3 < 32 * 3 * mat + extra + (1 << 16)
    assert lib.dash_workspace_bytes(0, 1024, 0, 4, 0) == 0 and lib.dash_workspace_bytes(4, 100, 0, 4, 0) == 0


def test_no_gpu_means_error_not_fallback(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    h = ctypes.c_void_p()
    assert lib.dash_create(ctypes.byref(h), 0, None) == 4            # DASH_ERR_HIP
    assert not h.value
    from paper_2602_02016_amd import Dash, DashError
    with pytest.raises(DashError):
        Dash(0)
    assert lib.dash_status_string(3).decode().startswith("workspace")
