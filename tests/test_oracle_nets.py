"""The oracle's layer chains against full-precision forwards and structural invariants."""
import numpy as np
import pytest

from oracle import nets, oracle as o
from workloads import calib, configs as cf, gen


def _f64_forward(layers, x, params):
    x = np.asarray(x, np.float64)
    for L, (w, b) in zip(layers, params):
        if L.kind == "conv":
            x = o.conv2d_f64(x, w, b, L.stride, L.pad, L.groups, L.relu)
            if L.pool_k:
                x = o.maxpool_f64(x, L.pool_k, L.pool_s)
        else:
            x = o.gemm_f64(x.reshape(x.shape[0], -1), w, b, L.relu)
    return x


@pytest.mark.parametrize("dtype,tol", [("int8", 0.08), ("int16", 1e-3)])
def test_lenet_quantized_tracks_full_precision(dtype, tol):
    x, params = cf.lenet_tensors(8)
    sc = calib.load()["lenet"][dtype]
    q = nets.run_int_chain(cf.LENET_LAYERS, x, params, sc["x"], sc["layers"], dtype)
    assert q.shape == (8, 10)
    real = o.dequantize(q, sc["layers"][-1]["y"], 0).astype(np.float64)
    ref = _f64_forward(cf.LENET_LAYERS, x, params)
    assert np.max(np.abs(real - ref)) <= tol * np.max(np.abs(ref))


def test_fp16_chain_tracks_full_precision():
    x, params = cf.lenet_tensors(4)
    y = nets.run_fp16_chain(cf.LENET_LAYERS, x, params)
    ref = _f64_forward(cf.LENET_LAYERS, x, params)
    assert np.max(np.abs(y - ref)) <= 5e-3 * np.max(np.abs(ref))


def _tiny_moe(dtype="int8"):
    layers = [cf.Conv("c", 6, 4, 3, 3, pad=1, groups=2, pool_k=3, pool_s=2), cf.FC("f", 5, 6 * 2 * 2)]
    E = 3
    params, scales = [], []
    for e in range(E):
        ps = [(gen.integers(100 + e, (6, 2, 3, 3), -100, 100), gen.integers(200 + e, (6,), -300, 300)),
              (gen.integers(300 + e, (5, 24), -100, 100), gen.integers(400 + e, (5,), -300, 300))]
        params.append(ps)
        scales.append([{"w": 0.01, "b": 0.0002, "y": 0.3 + 0.1 * e}, {"w": 0.02, "b": 0.006, "y": 1.5}])
    x = gen.integers(7, (10, 4, 5, 5), -128, 127)
    return layers, params, scales, x, E


def test_moe_all_to_one_expert_and_permutation_invariance():
    layers, params, scales, x, E = _tiny_moe()
    B = x.shape[0]
    for j in range(E):
        lg = gen.normal(j, (B, E))
        lg[:, j] += 50
        y, e_idx, counts = nets.moe_int(x, 0.02, lg, layers, params, scales, "int8")
        assert counts[j] == B
        # equals expert j evaluated on the whole batch at once
        a = nets.int_conv(x, 0, 0.02, params[j][0][0], 0, params[j][0][1], layers[0], scales[j][0], "int8")
        a = nets.int_fc(a.reshape(B, -1), 0, scales[j][0]["y"], params[j][1][0], 0, params[j][1][1],
                        layers[1], scales[j][1], "int8")
        assert np.array_equal(y, a)
    lg = gen.normal(9, (B, E))
    y, e_idx, counts = nets.moe_int(x, 0.02, lg, layers, params, scales, "int8")
    assert counts.sum() == B and len(set(e_idx.tolist())) > 1
    perm = gen.permutation(3, B)
    y2, e2, c2 = nets.moe_int(x[perm], 0.02, lg[perm], layers, params, scales, "int8")
    assert np.array_equal(y2, y[perm]) and np.array_equal(e2, e_idx[perm]) and np.array_equal(c2, counts)
