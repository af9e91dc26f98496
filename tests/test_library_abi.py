"""The C-ABI library: it loads, exports every symbol the header declares, and its
host-side argument checks work without a GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in ("fastserve.h", "fastserve_sched.h", "fastserve_kvm.h")]


@pytest.fixture(scope="module")
def fs():
    import paper_2305_05920_amd as fs
    if not os.path.exists(fs.LIB_PATH):
        from paper_2305_05920_amd import build
        build.build_library()
    fs.load_library()
    return fs


def declared_functions():
    text = "".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fs_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_function_is_exported(fs):
    names = declared_functions()
    assert "fs_pool_create" in names and "fs_kv_append" in names and "fs_decode_attention" in names
    lib = fs.load_library()
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"
    from paper_2305_05920_amd import kvm, sched
    assert sorted(fs.EXPORTS + sched.SCHED_EXPORTS + kvm.KVM_EXPORTS) == names, \
        "binding and headers disagree on the entry points"


def test_status_strings_and_version(fs):
    assert fs.strerror(0) == "ok"
    assert "table" in fs.strerror(fs.FS_ERR_BAD_TABLE)
    assert fs.strerror(-99) == "unknown status"
    assert fs.version().startswith("fastserve")


def test_host_side_argument_checks_need_no_gpu(fs):
    lib = fs.load_library()
    assert lib.fs_pool_block_bytes(None) == 0
    assert lib.fs_pool_destroy(None) == fs.FS_ERR_INVALID_ARG
    handle = ctypes.c_void_p()
    assert lib.fs_pool_create(None, ctypes.byref(handle)) == fs.FS_ERR_INVALID_ARG
    cfg = fs.fs_pool_config()
    cfg.dtype, cfg.num_heads, cfg.head_dim, cfg.block_size, cfg.num_blocks = 7, 4, 128, 16, 8
    assert lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)) == fs.FS_ERR_UNSUPPORTED
    cfg.dtype, cfg.head_dim = fs.FS_BF16, 96
    assert lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)) == fs.FS_ERR_UNSUPPORTED
    cfg.head_dim, cfg.block_size = 128, 32
    assert lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)) == fs.FS_ERR_UNSUPPORTED
    cfg.block_size, cfg.num_blocks = 16, 0
    assert lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)) == fs.FS_ERR_INVALID_ARG
    cfg.num_blocks, cfg.reserved = 8, 1
    assert lib.fs_pool_create(ctypes.byref(cfg), ctypes.byref(handle)) == fs.FS_ERR_INVALID_ARG
    assert lib.fs_kv_append(None, None, 1, None, 1, None, None, None) == fs.FS_ERR_INVALID_ARG
    assert lib.fs_decode_attention(None, None, None, 1, None, 1, 0, None, None) == fs.FS_ERR_INVALID_ARG
    assert lib.fs_pool_offload(None, None, None, 1, None) == fs.FS_ERR_INVALID_ARG
    assert not handle.value


def test_product_package_does_not_import_the_oracle(fs):
    import sys
    pkg = os.path.join(ROOT, "paper_2305_05920_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "fs_oracle" not in text, f
    otext = "".join(open(os.path.join(ROOT, "oracle", f)).read() for f in os.listdir(os.path.join(ROOT, "oracle"))
                    if f.endswith((".py", ".c")))
    assert "paper_2305_05920_amd" not in otext and "fastserve.h" not in otext


def test_pool_refuses_to_run_without_a_gpu(fs):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is visible")
    with pytest.raises(RuntimeError):
        fs.Pool("bf16", 4, 128, 8)
