"""The C-ABI library loads and exports every symbol the header declares, and rejects bad
arguments with error codes before touching the device (no GPU needed)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "pipe.h")
LIB = os.path.join(ROOT, "paper_2311_15806_amd", "libpipe_hip.so")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(LIB):
        pytest.fail("libpipe_hip.so is not built: run __graft_entry__.build() first")
    return C.CDLL(LIB)


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(pipe_[a-z0-9_]+)\s*\(", src)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"pipe_expand", "pipe_forward", "pipe_forward_acc", "pipe_forward_conv2d", "pipe_mlp_forward",
            "pipe_chain_forward", "pipe_chain_forward_conv", "pipe_expansion_order", "pipe_expansion_free", "pipe_strerror"} <= set(names)
    for n in names:
        assert hasattr(lib, n), "missing symbol " + n


def test_argument_errors_return_codes(lib):
    vp = C.c_void_p
    lib.pipe_expand.argtypes = [vp, C.c_int, C.c_int, C.c_int, C.c_int, C.c_float, C.c_int, vp, C.POINTER(vp)]
    lib.pipe_strerror.restype = C.c_char_p
    h = vp()
    fake = vp(256)          # never dereferenced: validation fails first
    EINVAL, ESHAPE = -1, -2
    assert lib.pipe_expand(None, 64, 64, 4, 2, 0.5, 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand(fake, 64, 64, 9, 2, 0.5, 16, None, C.byref(h)) == EINVAL      # bits
    assert lib.pipe_expand(fake, 64, 64, 1, 2, 0.5, 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand(fake, 64, 64, 4, 0, 0.5, 16, None, C.byref(h)) == EINVAL      # K
    assert lib.pipe_expand(fake, 64, 64, 4, 2, 0.0, 16, None, C.byref(h)) == EINVAL      # gamma
    assert lib.pipe_expand(fake, 64, 64, 4, 2, 1.5, 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand(fake, 60, 64, 4, 2, 0.5, 16, None, C.byref(h)) == ESHAPE      # out % group
    assert lib.pipe_expand(fake, 64, 64, 4, 2, 0.5, 8, None, C.byref(h)) == ESHAPE       # group % 16
    assert lib.pipe_expand(fake, 0, 64, 4, 2, 0.5, 16, None, C.byref(h)) == ESHAPE
    assert h.value is None
    assert lib.pipe_expand_conv2d(None, 64, 64, 3, 3, 4, 2, C.c_float(0.5), 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand_conv2d(fake, 64, 48, 3, 3, 4, 2, C.c_float(0.5), 16, None, C.byref(h)) == ESHAPE    # C % 64
    assert lib.pipe_expand_unstructured(None, 64, 64, 4, 2, C.c_float(0.5), 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand_unstructured(fake, 64, 64, 4, 2, C.c_float(1.5), 16, None, C.byref(h)) == EINVAL
    assert lib.pipe_expand_unstructured(fake, 60, 64, 4, 2, C.c_float(0.5), 16, None, C.byref(h)) == ESHAPE
    assert lib.pipe_expand_with_operator(fake, 64, 64, 4, 2, C.c_float(0.5), 16, None, None, fake, fake, fake, None, C.byref(h)) == EINVAL   # no operator
    assert lib.pipe_forward(None, None, 4, C.c_float(0), None, 0, None, 1, None, None) == EINVAL
    assert lib.pipe_chain_forward(None, 1, None, 4, C.c_float(0), None, 0, None, None, None) == EINVAL
    assert lib.pipe_chain_forward(fake, 0, None, 4, C.c_float(0), None, 0, None, None, None) == EINVAL
    assert lib.pipe_chain_forward_conv(None, 1, None, 1, 4, 4, C.c_float(0), None, 0, None, None, None) == EINVAL
    assert lib.pipe_chain_forward_asymmetric(None, 1, None, 1, None, 0, None, None, None) == EINVAL
    assert lib.pipe_chain_forward_conv_asymmetric(None, 1, None, 1, 4, 4, None, 0, None, None, None) == EINVAL
    assert lib.pipe_mlp_forward_asymmetric(None, None, 1, None, 1, None, 0, None, None, None, None, None) == EINVAL
    assert lib.pipe_mlp_forward_given_scales(None, None, 1, None, 1, C.c_float(1), None, None, 0, None, None, None, None, None) == EINVAL
    assert lib.pipe_spectral_norm(None, 4, 4, 3, None, None) == EINVAL
    assert lib.pipe_expansion_reconstruct(None, 1, None, None) == EINVAL
    assert lib.pipe_expansion_error_bound(None, None, None) == EINVAL
    lib.pipe_error_bound_U.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_double), C.c_int, C.POINTER(C.c_double)]
    s2, u2, U = (C.c_double * 2)(2.0, 4.0), (C.c_double * 2)(0.05, 0.01), C.c_double()
    assert lib.pipe_error_bound_U(s2, u2, 2, C.byref(U)) == 0 and abs(U.value - ((0.1 + 1) * (0.14 + 1) - 1)) < 1e-15
    assert lib.pipe_error_bound_U(s2, u2, 0, C.byref(U)) == EINVAL
    assert lib.pipe_expansion_order_norms(None, 3, None, None) == EINVAL
    assert lib.pipe_fold_batchnorm(None, None, None, None, None, None, C.c_float(1e-5), 4, 4, None, None, None) == EINVAL
    assert lib.pipe_forward_depthwise2d(None, None, 1, 4, 4, 4, 3, 3, 1, 1, 0, C.c_float(0), None, 0, None, 1, None, None) == EINVAL
    assert lib.pipe_forward_asymmetric(None, None, 4, None, 0, None, None, None) == EINVAL
    assert lib.pipe_forward_acc_asymmetric(None, None, 4, None, None, None, None, None) == EINVAL
    assert lib.pipe_forward_conv2d_asymmetric(None, None, 1, 4, 4, 4, 3, 3, 1, 1, 0, None, 0, None, None, None) == EINVAL
    assert lib.pipe_forward_conv2d_acc(None, None, 1, 4, 4, 4, 3, 3, 1, 1, 0, C.c_float(0), fake, None, None, None) == EINVAL
    assert lib.pipe_forward_conv2d_acc(fake, None, 1, 4, 4, 4, 3, 3, 1, 1, 0, C.c_float(0), None, None, None, None) == EINVAL   # no accumulator buffer
    assert lib.pipe_prepare(None, None, 0, 16, None) == EINVAL
    assert lib.pipe_prepare(fake, None, 0, 0, None) == EINVAL
    assert lib.pipe_prepare_mlp(None, None, 1, None, 0, 16, None) == EINVAL
    assert lib.pipe_prepare_chain(None, 1, 4, 1, 1, None, 0, None) == EINVAL
    assert lib.pipe_expansion_free(None) == 0
    assert lib.pipe_set_kernel(7) == EINVAL and lib.pipe_set_kernel(0) == 0
    assert lib.pipe_set_stream_split(-1) == EINVAL and lib.pipe_set_stream_split(0) == 0
    assert lib.pipe_set_decode_fusion(2) == EINVAL and lib.pipe_set_decode_fusion(1) == 0
    assert lib.pipe_set_decode_resident(3) == EINVAL and lib.pipe_set_decode_resident(1) == 0
    assert lib.pipe_set_resident_spin_limit(-1) == EINVAL and lib.pipe_set_resident_spin_limit(0) == 0
    assert lib.pipe_resident_status(None, None) == EINVAL
    assert lib.pipe_set_token_tile(48) == EINVAL and lib.pipe_set_token_tile(0) == 0
    assert lib.pipe_set_activation_bits(9) == EINVAL and lib.pipe_set_activation_bits(1) == EINVAL
    for code in (0, -1, -2, -3, -4, -5, -6):
        assert len(lib.pipe_strerror(code)) > 0


def test_binding_names_match_header():
    import paper_2311_15806_amd.binding as b
    for n in declared_functions():
        if n in ("pipe_strerror", "pipe_last_device_error", "pipe_expansion_free", "pipe_expansion_info"):
            continue      # reached through PipeError / Expansion
        assert hasattr(b, n), "binding lacks " + n


def test_product_never_reaches_the_checker():
    """The package (binding, workloads, build) holds no reference to the CPU checker, and the
    checker none to the package: they share only the seeded input generators, which hold no
    arithmetic of the method."""
    pkg = os.path.join(ROOT, "paper_2311_15806_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f), errors="ignore").read()
                assert "oracle" not in src.lower(), "%s mentions the checker" % f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith(".py"):
            src = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2311_15806_amd" not in src and "ctypes" not in src
    wl = open(os.path.join(pkg, "workloads.py")).read()
    for word in ("rint", "clip", "quantize(", "expand("):
        assert word not in wl, "the input generators must hold none of the method's arithmetic"
    bench = open(os.path.join(ROOT, "bench.py")).read()
    assert bench.count("from oracle import") == 1 and "if not args.no_cpu" in bench


def test_U_ens_and_predictor_size_rule_host_arithmetic():
    """The library's U_ens and K_1 rule are host arithmetic: checked here, without a GPU, against
    the hand-evaluated instances (the same file pins the checker)."""
    import json
    lib = C.CDLL(LIB)
    pd, pi = C.POINTER(C.c_double), C.POINTER(C.c_int)
    lib.pipe_error_bound_U_ens.argtypes = [pd, pd, C.c_int, C.c_int, pi, C.c_int, pd]
    lib.pipe_first_predictor_size.argtypes = [pd, pd, C.c_int, C.c_int, C.c_double, C.c_double, pi]
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "uens_worked.json")))

    def flat(rows):
        return None if rows is None else (C.c_double * (len(rows) * len(rows[0])))(*[float(v) for r in rows for v in r])

    U = C.c_double()
    for c in g["cases"]:
        L, K = len(c["norms"]), len(c["norms"][0])
        sp = (C.c_int * len(c["split"]))(*c["split"])
        assert lib.pipe_error_bound_U_ens(flat(c["norms"]), flat(c["lam"]), L, K, sp, len(c["split"]), C.byref(U)) == 0
        assert abs(U.value - c["U"]) <= 1e-12 * c["U"], c["name"]
    r = g["k1_rule"]
    norms, K = flat(r["norms"]), len(r["norms"][0])
    for K1, want in enumerate(r["U_by_K1"], start=1):
        sp = (C.c_int * 2)(K1, K - K1)
        assert lib.pipe_error_bound_U_ens(norms, None, 2, K, sp, 2, C.byref(U)) == 0 and abs(U.value - want) < 1e-12
    k1 = C.c_int()
    for q in r["queries"]:
        assert lib.pipe_first_predictor_size(norms, None, 2, K, q["logit_norm"], q["ratio"], C.byref(k1)) == 0
        assert k1.value == q["K1"], q
    bad = (C.c_int * 2)(1, 1)
    assert lib.pipe_error_bound_U_ens(norms, None, 2, K, bad, 2, C.byref(U)) == -5     # does not sum to K
    assert lib.pipe_error_bound_U_ens(norms, None, 2, K, None, 0, C.byref(U)) == 0     # one predictor
    assert abs(U.value - (4 + 1 + 0.25 + 0.0625) / 2) < 1e-12
