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


def test_create_reports_every_unsupported_configuration_as_shape_error():
    """Configuration checks run before anything touches the GPU."""
    from paper_2102_10485_amd import binding
    lib = binding.load_library()
    good = dict(cond_g=0, cond_d=0, z_dim=100, img_c=3, img_hw=32, g_h0=4, g_ch=[512, 256, 128], d_ch=[128, 256, 512])

    def status(n_models=4, n_labels=4, **changes):
        spec = dict(good)
        spec.update(changes)
        cfg = binding.make_config(spec, n_models, n_labels, 64)
        h = ctypes.c_void_p()
        return lib.gan_create(ctypes.byref(cfg), None, ctypes.byref(h))

    assert status(img_c=5) == binding.GAN_E_SHAPE                       # more than four image channels
    assert status(img_hw=48) == binding.GAN_E_SHAPE                     # g_h0 * 2^n_g != img_hw
    assert status(g_ch=[512, 256, 192]) == binding.GAN_E_SHAPE          # image-side layers take 64 or 128 feature channels
    assert status(d_ch=[256, 256, 512]) == binding.GAN_E_SHAPE
    assert status(g_ch=[2048, 256, 128]) == binding.GAN_E_SHAPE         # more than 1024 channels
    assert status(n_models=3, n_labels=4) == binding.GAN_E_SHAPE        # neither one model nor one per label
    assert status(cond_d=2) == binding.GAN_E_SHAPE                      # label maps must cover every label
    assert status(z_dim=0) == binding.GAN_E_SHAPE


def test_null_and_range_arguments_are_refused_on_the_host():
    from paper_2102_10485_amd import binding
    lib = binding.load_library()
    dbl = ctypes.c_double()
    assert lib.gan_generate(None, None, None, 1, None, 0) == binding.GAN_E_ARG
    assert lib.gan_sample(None, None, None, None, 1, None, None, 1) == binding.GAN_E_ARG
    assert lib.gan_anova_f(None, None, None, 1, ctypes.byref(dbl)) == binding.GAN_E_ARG
    assert lib.gan_get_losses(None, None, None, None) == binding.GAN_E_ARG
    assert lib.gan_probe_mfma(7, None, ctypes.byref(dbl)) == binding.GAN_E_ARG          # unknown precision
    assert lib.gan_probe_copy(100, None, ctypes.byref(dbl)) == binding.GAN_E_ARG        # below 1 MiB / not a multiple of 16
    assert lib.gan_probe_copy(1 << 20, None, None) == binding.GAN_E_ARG
