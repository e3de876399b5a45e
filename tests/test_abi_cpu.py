"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2505_16162_amd import binding, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_16162_amd.build import build_library
        build_library()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "knnssd.h")).read()
    declared = set(re.findall(r"\b(knnssd_[a-z_0-9]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_size_queries_and_shape_checks(lib):
    wl = synth.workload("llama13b")
    cfg = binding.make_cfg(wl.shape, 1000)
    kv = lib.knnssd_kvcache_bytes(ctypes.byref(cfg))
    # 40 blocks x (K and V) x 40 heads x 1552 positions x 128 x 2 bytes
    assert kv == 40 * 2 * 40 * wl.shape.max_seq * 128 * 2
    assert lib.knnssd_workspace_bytes(ctypes.byref(cfg)) > 16 * 32000 * 4
    assert lib.knnssd_workspace_bytes(None) == 0
    bad = binding.make_cfg(synth.small_shape("x", head_dim=48), 0)
    assert lib.knnssd_workspace_bytes(ctypes.byref(bad)) == 0
    bad2 = binding.make_cfg(synth.small_shape("x", n_heads=4, n_kv_heads=3), 0)
    assert lib.knnssd_workspace_bytes(ctypes.byref(bad2)) == 0


def test_null_arguments_are_rejected_without_a_device(lib):
    h = ctypes.c_void_p()
    cfg = binding.make_cfg(synth.workload("tiny").shape, 8)
    w = binding.Weights()
    assert lib.knnssd_create(ctypes.byref(cfg), ctypes.byref(w), None, 0, None, 0, None, ctypes.byref(h)) == -1
    assert lib.knnssd_create(None, None, None, 0, None, 0, None, ctypes.byref(h)) == -1
    assert lib.knnssd_destroy(None) == -1
    assert lib.knnssd_set_skipset(None, None) == -1
    assert lib.knnssd_set_anchors(None, None, 0, None, 1, 256, None, 1, 8) == -1
    assert lib.knnssd_draft_step(None, 0, 0, None, None) == -1
    assert lib.knnssd_verify(None, None, 0, 0, None, None, None) == -1
    assert lib.knnssd_generate(None, None, 0, None, None, None, None, None) == -1
    assert lib.knnssd_strerror(-3).decode().startswith("position")
    assert lib.knnssd_strerror(0).decode() == "ok"


def test_create_rejects_buffers_smaller_than_the_size_queries(lib):
    """The kernels index the caller's buffers by the layout of the cfg given to knnssd_create; a buffer sized
    for a different cfg (e.g. before weights_packed was set) must be refused before anything touches the device."""
    shape = synth.small_shape("sz", d_ffn=704, max_seq=160)
    cfg = binding.make_cfg(shape, 0)
    plain = lib.knnssd_workspace_bytes(ctypes.byref(cfg))
    assert lib.knnssd_pack_supported(ctypes.byref(cfg)) == 1
    cfg.weights_packed = 1
    packed = lib.knnssd_workspace_bytes(ctypes.byref(cfg))
    kv = lib.knnssd_kvcache_bytes(ctypes.byref(cfg))
    assert packed > plain > 0          # the stream-order path keeps all prompt rows of a prefill in its workspace
    h = ctypes.c_void_p()
    w = binding.Weights()
    fake = ctypes.c_void_p(0x100000)   # never dereferenced: the size check comes first
    assert lib.knnssd_create(ctypes.byref(cfg), ctypes.byref(w), fake, kv, fake, plain, None, ctypes.byref(h)) == -1
    assert lib.knnssd_create(ctypes.byref(cfg), ctypes.byref(w), fake, kv - 1, fake, packed, None, ctypes.byref(h)) == -1
    assert not h.value


def test_route_static_checks_its_arguments_before_touching_the_device(lib):
    """knnssd_route_static: every refusal below is decided on the host, in front of the first HIP call."""
    fake = ctypes.c_void_p(0x100000)
    odd = ctypes.c_void_p(0x100004)
    f = lib.knnssd_route_static
    assert f(None, fake, fake, 8, 256, None, fake) == -1
    assert f(fake, None, fake, 8, 256, None, fake) == -1
    assert f(fake, fake, None, 8, 256, None, fake) == -1
    assert f(fake, fake, fake, 8, 256, None, None) == -1
    assert f(odd, fake, fake, 8, 256, None, fake) == -1          # 16-byte alignment of query and anchors
    assert f(fake, odd, fake, 8, 256, None, fake) == -1
    assert f(fake, fake, fake, 8, 255, None, fake) == -2         # the scan reads 16-byte pieces of an anchor
    assert f(fake, fake, fake, 8, 0, None, fake) == -2
    assert f(fake, fake, fake, 0, 256, None, fake) == -3
    assert f(fake, fake, fake, 65537, 256, None, fake) == -3     # beyond KNNSSD_ROUTE_MAX_ANCHORS
    header = open(os.path.join(ROOT, "include", "knnssd.h")).read()
    assert "#define KNNSSD_ROUTE_MAX_ANCHORS 65536" in header


def test_stream_transition_is_a_host_call_with_argument_checks(lib):
    f = lib.knnssd_stream_next_domain
    assert f(2, 5, 0.0, 0.5, 0.5) == 2                  # r = 0: task by task
    assert f(2, 5, 1.0, 0.0, 0.0) == 0 and f(2, 5, 1.0, 0.0, 0.999999) == 4 and f(2, 5, 1.0, 0.0, 0.5) == 3   # never itself
    assert f(0, 1, 1.0, 0.0, 0.0) == 0
    assert f(5, 5, 0.5, 0.1, 0.1) == -3 and f(-1, 5, 0.5, 0.1, 0.1) == -3
    assert f(0, 0, 0.5, 0.1, 0.1) == -1
    assert f(0, 5, 1.5, 0.1, 0.1) == -3 and f(0, 5, 0.5, 1.0, 0.1) == -3 and f(0, 5, 0.5, 0.1, -0.1) == -3
