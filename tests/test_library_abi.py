"""Host-side checks that need no GPU: the built library loads, exports every entry point the
header declares, and validates configurations."""
import ctypes as C
import os
import re

import pytest

from paper_2402_18994_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2402_18994_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "snn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(snn_[a-z_]+)\s*\(", text)))


def test_every_declared_entry_point_is_exported(lib):
    names = declared_functions()
    assert {"snn_init", "snn_forward", "snn_backward", "snn_sgd_step"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c():
    src = os.path.join(ROOT, "_build_hdr_check.c")
    try:
        open(src, "w").write('#include "include/snn.h"\nint main(void){snn_config c; (void)c; return SNN_OK;}\n')
        assert os.system(f"cd {ROOT} && gcc -std=c99 -Wall -Werror -fsyntax-only {src}") == 0
    finally:
        os.remove(src)


def ws(lib, **kw):
    d = dict(T=8, B=4, sizes=(10, 6, 3), recurrent=(0,), beta=(0.9, 0.9), theta=1.0,
             surrogate="superspike", slope=25.0, precision="fp32")
    d.update(kw)
    return binding.workspace_bytes(**d)


def test_workspace_size_and_validation(lib):
    n = ws(lib)
    assert n > 0 and n % 256 == 0
    assert ws(lib, T=16) > n
    assert ws(lib, recurrent=(1,)) > n
    assert ws(lib, loss="integral") == n
    for s_ in ("boxcar", "ste"):
        assert ws(lib, surrogate=s_) == n
    for bad in (dict(T=0), dict(B=-1), dict(sizes=(10, 0, 3)), dict(beta=(0.9, 1.5)), dict(theta=0.0),
                dict(slope=-1.0), dict(surrogate=9), dict(precision=5), dict(loss=7),
                dict(sizes=(10, 3), beta=(0.9,), recurrent=())):
        with pytest.raises(binding.SnnError) as e:
            ws(lib, **bad)
        assert e.value.status == 2, bad
    # NULL pointers
    assert lib.snn_workspace_bytes(None, None) == 1
    assert b"NULL" in lib.snn_last_error(None)
    assert lib.snn_forward(None, None, None, None) == 1
    assert lib.snn_forward_packed(None, None, None, None) == 1
    assert lib.snn_backward(None) == 1
    assert lib.snn_sgd_step(None, C.c_float(0.1)) == 1
    assert lib.snn_destroy(None) == 0


def test_layer_count_limit(lib):
    """SNN_MAX_LAYERS = 12 weight matrices are admitted (with recurrent layers and trained decays
    that is 35 gradient reductions per backward pass, which the job lists hold), 13 are not."""
    hdr = open(os.path.join(ROOT, "include", "snn.h")).read()
    assert int(re.search(r"#define SNN_MAX_LAYERS (\d+)", hdr).group(1)) == 12
    for L, ok in ((12, True), (13, False)):
        kw = dict(sizes=(10,) + (8,) * (L - 1) + (3,), recurrent=(1,) * (L - 1), beta=(0.9,) * L)
        if ok:
            assert ws(lib, **kw) > 0
        else:
            with pytest.raises(binding.SnnError) as e:
                ws(lib, **kw)
            assert e.value.status == 2
    # the entry point without allocation validates its arguments before touching a device
    assert lib.snn_weight_grad_static(None, None, None, C.c_int64(8), 8, 8, None) == 1
    assert lib.snn_set_option(None, 0, 0) == 1 and lib.snn_get_option(None, 0, None) == 1


def test_headline_workspace_fits_one_gpu(lib):
    import workloads
    for name in workloads.CONFIG_ORDER:
        wl = workloads.CONFIGS[name]
        n = binding.workspace_bytes(wl.T, wl.B, wl.sizes, wl.recurrent, wl.beta, wl.theta, wl.surrogate,
                                    wl.slope, wl.precision)
        assert n < 200 * 2 ** 30, (name, n)
