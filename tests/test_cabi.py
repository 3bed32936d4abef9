"""The C-ABI library loads and exports every function include/gan.h declares (no compute without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gan_[a-z_0-9]+)\s*\(", text)))


def test_header_lists_the_boundary():
    names = declared_functions()
    for must in ("gan_create", "gan_train_step", "gan_generate", "gan_get_losses", "gan_destroy"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2102_10485_amd import binding
    if not os.path.exists(binding.lib_path()):
        from paper_2102_10485_amd import build
        build.build()
    lib = ctypes.CDLL(binding.lib_path())
    for name in declared_functions():
        assert hasattr(lib, name), name


def test_config_struct_matches_header_size():
    from paper_2102_10485_amd import binding
    # 4 + 4*10 + 4*8 + 4 + 4*8 + 4 + 4*10 + (pad) + 8
    assert ctypes.sizeof(binding.GanConfig) % 8 == 0
    cfg = binding.make_config(dict(cond_g=0, cond_d=0, z_dim=100, img_c=3, img_hw=32, g_h0=4, g_ch=[512, 256, 128],
                                   d_ch=[128, 256, 512]), 100, 100, 6400, binding.BF16)
    assert cfg.struct_size == ctypes.sizeof(binding.GanConfig) and cfg.n_g == 3 and cfg.d_ch[2] == 512


def test_create_rejects_bad_arguments_without_a_gpu():
    from paper_2102_10485_amd import binding
    lib = binding.load_library()
    spec = dict(cond_g=0, cond_d=0, z_dim=100, img_c=3, img_hw=32, g_h0=4, g_ch=[512, 256, 100], d_ch=[128, 256, 512])
    cfg = binding.make_config(spec, 4, 4, 64)
    h = ctypes.c_void_p()
    assert lib.gan_create(ctypes.byref(cfg), None, ctypes.byref(h)) == binding.GAN_E_SHAPE   # 100 channels
    cfg.struct_size = 12
    assert lib.gan_create(ctypes.byref(cfg), None, ctypes.byref(h)) == binding.GAN_E_ARG
    assert lib.gan_train_step(None, None, None, None, 4) == binding.GAN_E_ARG
