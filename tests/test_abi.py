"""Host-side checks of the C ABI: the library loads, exports what include/bls.h declares, and
the model layout matches the tensor order the synthetic weight generator uses."""
import ctypes
import os
import re

import numpy as np
import pytest

import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "bls.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{}]*\)\s*;", text)))


def test_library_exports_every_declared_symbol():
    import paper_2508_08540_amd as bls
    names = _declared_functions()
    assert set(names) == set(bls.DECLARED_SYMBOLS)
    raw = ctypes.CDLL(bls.library_path())
    for n in names:
        assert hasattr(raw, n), n


def test_layout_matches_generator_order_and_counts():
    import paper_2508_08540_amd as bls
    m = bls.Model.resnet_cifar()
    assert m.num_params == 269722 and m.num_buffers == 1376
    p_specs, b_specs = synth.resnet_tensor_specs()
    assert [(t["name"], t["shape"]) for t in m.tensors if not t["is_buffer"]] == p_specs
    assert [(t["name"], t["shape"]) for t in m.tensors if t["is_buffer"]] == b_specs
    mlp = bls.Model.mlp()
    assert mlp.num_params == 394634 and mlp.num_buffers == 0
    assert [(t["name"], t["shape"]) for t in mlp.tensors] == synth.mlp_tensor_specs()
    p, b = synth.resnet_init(1)
    flat = m.pack(p)
    back = m.unpack(flat)
    for k in p:
        np.testing.assert_array_equal(back[k], p[k])
    with pytest.raises(bls.BlsError):
        bls.Model.resnet_cifar(widths=(16, 24, 64))


def test_sequence_model_layout_and_rejected_descriptions():
    import paper_2508_08540_amd as bls
    m = bls.Model.transformer()
    assert m.num_params == 51747840 and m.num_buffers == 0
    assert [(t["name"], t["shape"]) for t in m.tensors] == [(n, tuple(s)) for n, s in synth.transformer_tensor_specs()]
    small = bls.Model.transformer(50, 8, 16, 2, 32, 2)
    assert [(t["name"], t["shape"]) for t in small.tensors] == [(n, tuple(s)) for n, s in synth.transformer_tensor_specs(50, 8, 16, 32, 2)]
    for bad in [dict(d_model=18), dict(heads=3), dict(seq_len=2048), dict(layers=0), dict(d_ff=30), dict(vocab=1)]:
        with pytest.raises(bls.BlsError):
            bls.Model.transformer(**bad)


def test_workspace_query():
    """Scratch sizes are a host-side function of the model and the batch: they grow with the training batch, stop growing
    once a pool is scored in chunks, and bad arguments are refused."""
    import paper_2508_08540_amd as bls
    for m, chunk in ((bls.Model.mlp(), 2048), (bls.Model.resnet_cifar(), 2048), (bls.Model.wide_resnet(act_dtype="bf16"), 1024),
                     (bls.Model.transformer(act_dtype="bf16"), 512), (bls.Model.transformer(), 256)):
        train = [m.workspace_bytes(n, True) for n in (16, 32, 64)]
        assert 0 < train[0] < train[1] < train[2]
        assert m.workspace_bytes(chunk // 2, False) < m.workspace_bytes(chunk, False) == m.workspace_bytes(4 * chunk, False)
        for bad in (0, -3, 1 << 25):
            with pytest.raises(bls.BlsError):
                m.workspace_bytes(bad, True)


def test_weights_from_tau_host_helper():
    import paper_2508_08540_amd as bls
    w = bls.weights_from_tau([32] * 8 + [16] * 2)
    np.testing.assert_array_equal(w, np.array([1 / 9] * 8 + [1 / 18] * 2, dtype=np.float32))
    with pytest.raises(bls.BlsError):
        bls.weights_from_tau([0, 0])


def test_epoch_allocation_and_worker_share_match_the_oracle():
    import oracle
    import paper_2508_08540_amd as bls
    for N, tf, pf, ts, ps, lam in [(50000, 32, 8, 1, 2, 1.0), (50000, 32, 8, 4, 2, 0.5), (100000, 32, 8, 1, 2, 0.25),
                                   (7, 3, 2, 1, 1, 0.5), (0, 1, 1, 1, 1, 1.0), (12345, 5, 3, 0, 0, 0.1)]:
        assert bls.epoch_allocation(N, tf, pf, ts, ps, lam) == oracle.allocation(N, tf, pf, ts, ps, lam)
    ranked = list(range(23))
    for P in (1, 2, 5, 23, 30):
        parts = oracle.deal(ranked, P)
        off = 0
        for p in range(P):
            assert bls.worker_share(len(ranked), P, p) == (off, len(parts[p]))
            off += len(parts[p])
