"""The C-ABI library loads without a GPU, exports every function the header declares, and its
host-side logic (status strings, workspace sizing, argument validation) behaves as documented."""
import ctypes
import os
import re

import pytest

from paper_2410_18035_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "milora.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(milora_[a-z_]+)\s*\(", text)))


def test_header_and_binding_name_the_same_entry_points():
    assert declared_functions() == sorted(mb.EXPORTS)


def test_library_exports_every_declared_symbol():
    L = mb.lib()
    for name in declared_functions():
        assert hasattr(L, name), f"{name} is declared in include/milora.h but not exported"


def test_status_strings_and_version():
    assert "gfx950" in mb.version()
    for code in (0, -1, -2, -3, -4, -5):
        assert mb.status_string(code) != "unknown status"
    assert mb.status_string(-99) == "unknown status"
    assert mb.last_hip_error() == 0


def test_workspace_sizes_are_monotone_and_reject_bad_sizes():
    assert mb.route_workspace_bytes(0, 4096, 100) == 0
    assert mb.route_workspace_bytes(32, 4096, 8192) >= 32 * 4096 * 4
    a = mb.layer_decode_workspace_bytes(16, 4096, 11008, 32)
    b = mb.layer_decode_workspace_bytes(32, 4096, 11008, 32)
    assert 0 < a < b
    # above 32 rows the workspace also holds the wide-batch kernel's tables: two halves of (256 workgroups + column
    # groups of the widest level) segments, each 12 tiles x the row tiles (4 up to 64 rows, 8 above) of 1 KiB partial
    # sums, a flag and the rows' sums of squares; 11008 / 16 gate/up pairs in groups of 6; and the LoRA term tiles
    # (1 KiB per tile and row tile: 2 * 688 gate/up tiles + 256 of o or down) with their flags
    c = mb.layer_decode_workspace_bytes(33, 4096, 11008, 32)
    segs = 2 * (256 + 115)
    lora_tiles = (2 * 688 + 256) * 4 * 1024
    assert segs * (48 * 1024 + 64 * 4 + 4) + lora_tiles <= c <= segs * (48 * 1024 + 64 * 4 + 4) + lora_tiles + (1 << 23)
    c = mb.layer_decode_workspace_bytes(65, 4096, 11008, 32)
    segs = 2 * (256 + 115)
    lora_tiles = (2 * 688 + 256) * 8 * 1024
    assert segs * (96 * 1024 + 128 * 4 + 4) + lora_tiles <= c <= segs * (96 * 1024 + 128 * 4 + 4) + lora_tiles + (1 << 23)
    assert mb.layer_decode_workspace_bytes(128, 4096, 11008, 32) >= c
    assert mb.layer_decode_workspace_bytes(129, 4096, 11008, 32) == 0  # beyond the decode batch limit
    assert mb.routed_linear_workspace_bytes(32768, 4096, 4096, 32) >= 32768 * 32 * 4


def test_kernel_choice_of_the_routed_linear():
    import torch

    k = mb.milora_routed_linear_kernel
    assert k(32, 4096, 4096, torch.bfloat16, mb.W_PACKED) == mb.KERNEL_STREAM
    assert k(32768, 4096, 11008, torch.bfloat16, mb.W_PACKED) == mb.KERNEL_STREAM
    assert k(32768, 4096, 11008, torch.bfloat16) == mb.KERNEL_TILES
    assert k(32768, 11008, 4096, torch.bfloat16) == mb.KERNEL_TILES
    assert k(64, 64, 16, torch.bfloat16) == mb.KERNEL_TILES
    assert k(63, 64, 16, torch.bfloat16) == mb.KERNEL_GENERIC  # few rows
    assert k(700, 96, 528, torch.bfloat16) == mb.KERNEL_GENERIC  # reduction not a multiple of 64
    assert k(700, 192, 520, torch.bfloat16) == mb.KERNEL_GENERIC  # width not a multiple of 16
    assert k(700, 192, 528, torch.float32) == mb.KERNEL_GENERIC
    assert k(1 << 20, 4096, 4096, torch.bfloat16) == mb.KERNEL_TILES  # in row slices with 32-bit byte offsets
    assert k(32, 4096, 4096, torch.float32, mb.W_PACKED) == -3
    assert k(0, 8, 8, torch.float32) == -1 and k(8, 8, 8, torch.float32, 5) == -1


def test_argument_validation_happens_before_any_device_work():
    L = mb.lib()
    null = ctypes.c_void_p(None)
    # null tensors
    assert L.milora_route(null, 10, 8, 0, null, null, null, 1, 1, null, 0, 0, null, None, 1, null, null, null, 0, null) == -1
    ad = mb._Adapters(1, 8, 0, 0, 0)
    assert L.milora_routed_linear(null, 1, 8, 8, 0, null, null, 0, null, ctypes.byref(ad), 0, null, null, 1, null,
                                  null, 0, null) == -1
    lw = mb._LayerWeights()
    assert L.milora_layer_decode(null, 1, 8, 8, 0, ctypes.byref(lw), ctypes.byref(ad), null, null, 0, null, null,
                                 null, null, 0, null) == -1
    assert L.milora_pack_weight(null, null, 32, 16, null) == -1
    # fake non-null pointers never get dereferenced on these paths: bad enum, bad site, missing workspace
    p = ctypes.c_void_p(0x1000)
    assert L.milora_route(p, 10, 8, 7, p, p, p, 1, 1, p, 0, 0, null, None, 1, p, null, p, 1 << 20, null) == -1  # dtype 7
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 4, 0, null, None, 1, p, null, p, 1 << 20, null) == -1  # pool 4
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 3, 0, null, None, 1, p, null, p, 1 << 20, null) == -1  # no w_sa
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 0, 4, null, None, 1, p, null, p, 1 << 20, null) == -1  # no coefficients
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 0, 0, null, None, 7, p, null, p, 1 << 20, null) == -1  # top_k 7
    assert L.milora_route(p, 10, 9000, 0, p, p, p, 1, 1, p, 3, 0, p, None, 1, p, null, p, 1 << 30, null) == -2  # d too large
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 0, 0, null, None, 1, p, null, null, 0, null) == -5  # no workspace
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 1, 0, null, None, 1, p, null, null, 0, null) == -5  # last-token pooling needs one too
    assert L.milora_route(p, 10, 8, 0, p, p, p, 1, 1, p, 0, 0, null, None, 1, p, null, p, 16, null) == -5  # too small
    out = ctypes.c_double(0.0)
    assert L.milora_measure_matrix_rate(4, 10, p, 1 << 30, ctypes.byref(out), null) == -1  # no such instruction shape
    assert L.milora_measure_matrix_rate(1, 0, p, 1 << 30, ctypes.byref(out), null) == -1  # no iterations
    assert L.milora_measure_matrix_rate(1, 10, null, 0, ctypes.byref(out), null) == -5  # no workspace
    ad = mb._Adapters(1, 8, 0x1000, 0x1000, 0x1000)
    assert L.milora_routed_linear(p, 1, 8, 8, 0, null, p, 0, null, ctypes.byref(ad), 9, p, p, 1, p, p, 1 << 20,
                                  null) == -1  # site 9
    assert L.milora_routed_linear(p, 2, 8, 8, 0, null, p, 0, null, ctypes.byref(ad), 0, p, p, 1, p, p, 1 << 20,
                                  null) == -1  # M != B without a row map
    ad_big = mb._Adapters(1, 1024, 0x1000, 0x1000, 0x1000)
    assert L.milora_routed_linear(p, 1, 8, 8, 0, null, p, 0, null, ctypes.byref(ad_big), 0, p, p, 1, p, p, 1 << 20,
                                  null) == -2  # rank limit
    assert L.milora_routed_linear(p, 1, 8, 8, 1, null, p, 1, null, ctypes.byref(ad), 0, p, p, 1, p, p, 1 << 20,
                                  null) == -3  # packed fp32
    assert L.milora_routed_linear(p, 1, 8, 8, 0, null, p, 0, null, ctypes.byref(ad), 0, p, p, 1, p, null, 0,
                                  null) == -5
    for m in range(7):
        lw.W[m] = 0x1000
    lw.layout = 1
    assert L.milora_layer_decode(p, 200, 64, 64, 0, ctypes.byref(lw), ctypes.byref(ad), p, p, 0, null, p, null, p,
                                 1 << 30, null) == -2  # batch limit
    assert L.milora_layer_decode(p, 4, 64, 64, 1, ctypes.byref(lw), ctypes.byref(ad), p, p, 0, null, p, null, p,
                                 1 << 30, null) == -3  # packed fp32
    assert L.milora_layer_decode(p, 4, 64, 64, 0, ctypes.byref(lw), ctypes.byref(ad), p, p, 8, null, p, null, p,
                                 1 << 30, null) == -1  # unknown flag
    assert L.milora_pack_weight(p, p, 33, 16, null) == -3


def test_binding_refuses_host_tensors():
    import torch

    with pytest.raises(ValueError):
        mb._dev(torch.zeros(4))
