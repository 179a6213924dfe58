"""CPU checks of the synthetic workloads: the shape recipes add up to the parameter counts they stand for (the five
benchmark configurations and the models of the paper's Table 1), and the generators are deterministic in their seeds."""
import numpy as np

import workloads
from workloads import shapes


def test_shape_recipes_add_up():
    expect = {
        "resnet50": (shapes.resnet50(), 25_557_032, 161),
        "lstm_lm": (shapes.lstm_lm(), 66_034_000, 9),          # Table 1: LSTM-PTB
        "vgg16": (shapes.vgg16(), 138_357_544, 32),
        "transformer": (shapes.transformer(), 1_500_000_000, None),
        "fnn3": (shapes.fnn3(), 199_210, 6),                    # Table 1: FNN-3
        "resnet20": (shapes.resnet20(), 269_722, 59),           # Table 1: ResNet-20
        "vgg16_cifar": (shapes.vgg16_cifar(), 14_728_266, 54),  # Table 1: VGG-16
    }
    for name, (tensors, total, count) in expect.items():
        assert shapes.total(tensors) == total, name
        assert count is None or len(tensors) == count, name
        assert all(numel > 0 for _, numel in tensors), name
        offs = shapes.offsets(tensors)
        assert offs[0] == 0 and all(offs[k + 1] == offs[k] + tensors[k][1] for k in range(len(tensors) - 1)), name
    assert shapes.total(shapes.transformer(truncate_to=None)) == 1_557_611_200
    assert [workloads.FULL[k]().n for k in (1, 2, 3, 4, 5)] == [1_048_576, 25_557_032, 66_034_000, 138_357_544, 1_500_000_000]
    assert [workloads.FULL[k]().num_workers for k in (1, 2, 3, 4, 5)] == [4, 8, 8, 16, 4]


def test_generators_are_deterministic_and_per_worker():
    for wl in [workloads.small(k) for k in (1, 2, 3, 4, 5)] + [workloads.table1("fnn3")]:
        a, b = wl.gradient(0, 0).numpy(), wl.gradient(0, 0).numpy()
        assert np.array_equal(a, b), wl.name
        assert not np.array_equal(a, wl.gradient(1, 0).numpy()), wl.name   # another worker
        assert not np.array_equal(a, wl.gradient(0, 1).numpy()), wl.name   # another step
        assert np.array_equal(wl.weights().numpy(), wl.weights().numpy())
        assert np.isfinite(a).all() and abs(float(a.mean())) < 10 * float(a.std()) / np.sqrt(a.size) + 1e-12, wl.name
    assert not workloads.FULL[1]().initial_error(0).any()
