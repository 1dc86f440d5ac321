"""Host logic of bench.py: the algorithmic flop and byte counts its roofline figures are built on."""
import importlib.util
import os

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench():
    spec = importlib.util.spec_from_file_location("_bench", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_resnet_flops_by_enumeration():
    b = _bench()
    # ResNet8 on 8x8 images: stem 3->16 at 8x8; 16->16, 16->16 at 8x8; 16->32 (stride 2), 32->32 at 4x4;
    # 32->64 (stride 2), 64->64 at 2x2.  2 flop per multiply-add, 9 taps.
    macs = 9 * (3 * 16 * 64 + 2 * 16 * 16 * 64 + (16 * 32 + 32 * 32) * 16 + (32 * 64 + 64 * 64) * 4)
    assert b.resnet_conv_flops((16, 32, 64), 1, 8, 3) == 2 * macs


def test_input_gradient_bytes_by_enumeration():
    b = _bench()
    # Same net, batch 2, 4-byte elements.  Layers above the stem as (c_in, c_out, h_in, h_out); t = elements of a tensor.
    B, elt = 2, 4
    t = lambda c, h: B * h * h * c
    total = 0
    # block 1 (16 -> 16 at 8x8): first layer of the block
    total += 2 * t(16, 8) + t(16, 8) + 3 * t(16, 8) + 9 * 16 * 16 + t(16, 8)        # dout,y | dy | a',y',dx | w | shortcut grad
    # block 1: second layer (the gradient it receives doubles as the shortcut gradient: nothing extra is written)
    total += 2 * t(16, 8) + t(16, 8) + 3 * t(16, 8) + 9 * 16 * 16
    # block 2 (16 -> 32, stride 2): first layer; its shortcut gradient covers the block's 4x4 output positions, 16 channels
    total += 2 * t(32, 4) + t(32, 4) + 3 * t(16, 8) + 9 * 16 * 32 + B * 4 * 4 * 16
    total += 2 * t(32, 4) + t(32, 4) + 3 * t(32, 4) + 9 * 32 * 32
    # block 3 (32 -> 64, stride 2); the top layer reads a finished dy instead of computing it
    total += 2 * t(64, 2) + t(64, 2) + 3 * t(32, 4) + 9 * 32 * 64 + B * 2 * 2 * 32
    total += t(64, 2) + 3 * t(64, 2) + 9 * 64 * 64
    assert b.resnet_dgrad_bytes((16, 32, 64), 1, 8, B, elt) == total * elt
