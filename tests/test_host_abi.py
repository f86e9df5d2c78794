"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, sizes the paper's network correctly and rejects bad arguments
without touching a GPU."""
import ctypes as C
import os
import re

import pytest

import synthetic_inputs as S

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_1412_2302_amd import binding
    return binding


def test_library_exports_every_declared_symbol(B):
    hdr = open(os.path.join(ROOT, "include", "alexnet.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(alexnet_[a-z0-9_]+)\s*\(", hdr))
    assert len(names) >= 25
    lib = C.CDLL(B.LIB_PATH)
    missing = [n for n in sorted(names) if not hasattr(lib, n)]
    assert not missing, missing
    assert set(B.EXPORTS) == names
    assert "gfx950" in B.version()


def test_query_sizes_the_full_network(B):
    cfg = B.make_config(S.ALEXNET, 128)
    n, ws = B.query(cfg)
    assert n == 60965224  # 2,332,704 conv + 58,621,952 dense weights + 10,568 biases
    assert ws % 256 == 0 and 1 << 30 < ws < 16 << 30
    n_mini, _ = B.query(B.make_config(S.MINI, 4))
    assert n_mini == 16*3*49 + 32*8*25 + 48*32*9 + 48*24*9 + 32*24*9 + 128*256 + 256*256 + 256*10 + (16+32+48+48+32+256+256+10)


def test_bad_arguments_are_reported_not_crashed(B):
    lib = C.CDLL(B.LIB_PATH)
    n, w = C.c_size_t(), C.c_size_t()
    lib.alexnet_query.restype = C.c_int
    assert lib.alexnet_query(None, C.byref(n), C.byref(w)) == B.EINVAL
    assert "null" in B.last_error()
    cfg = B.make_config(S.MINI, 4)
    cfg.conv[1].groups = 3  # 16 input channels are not divisible by 3
    with pytest.raises(B.AlexNetError) as e:
        B.query(cfg)
    assert e.value.code == B.ESHAPE and "conv2" in str(e.value)
    cfg = B.make_config(S.MINI, 4); cfg.crop_h = cfg.crop_w = 9; cfg.raw_h = cfg.raw_w = 9
    with pytest.raises(B.AlexNetError) as e:
        B.query(cfg)
    assert e.value.code == B.ESHAPE
    cfg = B.make_config(S.MINI, 0)
    with pytest.raises(B.AlexNetError):
        B.query(cfg)
    B.query(B.make_config(S.MINI, 4, precision=1))  # bf16 products are a valid configuration
    # maximum sizes: every tensor must stay below 2 GiB (32-bit byte offsets in the kernels)
    B.query(B.make_config(S.ALEXNET, 1024))          # conv1 activations: 1.19 GB
    with pytest.raises(B.AlexNetError) as e:
        B.query(B.make_config(S.ALEXNET, 2048))      # 2.38 GB
    assert e.value.code == B.ESHAPE and "2 GiB" in str(e.value)
    cfg = B.make_config(S.MINI, 4, precision=2)
    with pytest.raises(B.AlexNetError) as e:
        B.query(cfg)
    assert e.value.code == B.ENOTIMPL
    cfg = B.make_config(S.MINI, 4); cfg.lrn_n = 4
    with pytest.raises(B.AlexNetError) as e:
        B.query(cfg)
    assert e.value.code == B.EINVAL
    # flags: the direct-convolution choice is part of the configuration (it changes the workspace), unknown bits are refused
    _, ws_default = B.query(B.make_config(S.ALEXNET, 128))
    _, ws_direct = B.query(B.make_config(S.ALEXNET, 128, flags=B.FLAG_DIRECT_CONV))
    assert ws_direct < ws_default
    with pytest.raises(B.AlexNetError) as e:
        B.query(B.make_config(S.MINI, 4, flags=2))
    assert e.value.code == B.EINVAL and "flags" in str(e.value)
    # null handles / pointers on calls that would otherwise enqueue work
    for fn, args in [("alexnet_train_step", (None, 0, None, 0, None, None)),
                     ("alexnet_average_replicas", (None, None, None)),
                     ("alexnet_forward", (None, None, None, None)),
                     ("alexnet_preprocess", (None, None, None, 0, 0, None))]:
        assert getattr(B._lib, fn)(*args) == B.EINVAL
    # create refuses unaligned device pointers before any GPU work
    cfg = B.make_config(S.MINI, 4)
    h = C.c_void_p()
    rc = B._lib.alexnet_create(C.byref(cfg), C.c_void_p(0x1001), C.c_void_p(0x2000), C.c_void_p(0x3000), 1 << 30,
                               None, C.byref(h))
    assert rc == B.EALIGN


def test_binding_refuses_tensors_the_library_would_read_past(B):
    """The binding hands bare pointers to the library, so it checks place, type, layout and size first.  The
    checks run before any library call: a stand-in object with the fields they read is enough here."""
    import torch

    need = B._need
    with pytest.raises(TypeError):
        need([1, 2, 3], torch.int32, 3, "labels")
    with pytest.raises(ValueError, match="device tensor"):
        need(torch.zeros(4, dtype=torch.int32), torch.int32, 4, "labels")  # a host tensor

    class Net:  # geometry helpers of AlexNet without creating a handle
        workload, batch = S.MIDI, 5
        _conv_elems = B.AlexNet._conv_elems
        _raw_elems = B.AlexNet._raw_elems
        _input_elems = B.AlexNet._input_elems

    n = Net()
    assert n._raw_elems() == 3 * 80 * 80 and n._input_elems() == 5 * 3 * 67 * 67
    # midi: 67 -> conv1(11, s4) 15 -> pool 7 -> conv2(5, p2, g2) 7 -> pool 3 -> conv3 3
    assert n._conv_elems(1) == (5 * 67 * 67 * 3, 5 * 15 * 15 * 24, 24 * 3 * 121, 24)
    assert n._conv_elems(2) == (5 * 7 * 7 * 24, 5 * 7 * 7 * 40, 40 * 12 * 25, 40)
    assert n._conv_elems(3) == (5 * 3 * 3 * 40, 5 * 3 * 3 * 72, 72 * 40 * 9, 72)
    with pytest.raises(ValueError):
        n._conv_elems(6)
