"""The seeded input generator: deterministic, coordinate-keyed, N(0,1), exact bf16 round trip."""
import numpy as np

from paper_2405_07719_amd import inputs


def test_values_depend_only_on_coordinates():
    full = inputs.tensor_at(1001, inputs.TENSOR_K, 2, np.arange(64), np.arange(8), 16)
    part = inputs.tensor_at(1001, inputs.TENSOR_K, 2, np.array([5, 63, 17]), np.array([6, 1]), 16)
    assert np.array_equal(part, full[:, [5, 63, 17]][:, :, [6, 1]])
    other = inputs.tensor_at(1001, inputs.TENSOR_V, 2, np.arange(64), np.arange(8), 16)
    assert not np.array_equal(full, other)
    again = inputs.tensor_at(1001, inputs.TENSOR_K, 2, np.arange(64), np.arange(8), 16)
    assert np.array_equal(full, again)


def test_distribution_is_standard_normal():
    x = inputs.tensor_at(3, inputs.TENSOR_Q, 1, np.arange(4096), np.arange(4), 64).ravel()
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1.0) < 5e-3
    assert abs(np.mean(x ** 3)) < 2e-2 and abs(np.mean(x ** 4) - 3.0) < 5e-2
    # neighbouring coordinates are uncorrelated
    y = x.reshape(-1, 64)
    assert abs(np.corrcoef(y[:, 0], y[:, 1])[0, 1]) < 2e-2
    assert abs(np.corrcoef(y[:-1, 0], y[1:, 0])[0, 1]) < 2e-2


def test_bf16_round_trip_and_rounding():
    x = np.array([1.0, 1.00390625, 1.01171875, -2.5, 0.0, 3.140625, 1e-3], dtype=np.float64)
    bits = inputs.to_bf16_bits(x)
    back = inputs.from_bf16_bits(bits)
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to even (1.0); 1 + 3*2^-8 ties up to 1 + 2^-6
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625
    assert back[3] == -2.5 and back[4] == 0.0 and back[5] == 3.140625
    assert abs(back[6] - 1e-3) <= 1e-3 * 2.0 ** -8
    assert np.array_equal(inputs.to_bf16_bits(back), bits)      # idempotent
