"""Which kernel, rows per workgroup and split each layer of the five baseline configurations takes, on a 256-CU device,
through the C ABI's plan query (host code only: no GPU needed).  A change of the launch planner shows up here."""
import pytest

QUAD, XMAJOR, FAST, GENERIC, ROWS = 3, 2, 1, 0, -1


@pytest.fixture(scope="module")
def plan():
    from paper_2203_04071_amd import binding as B
    B.load()
    return lambda *a: B.adapt_plan_packed(*a, 256)


def test_headline_layer_runs_on_the_quad_kernel_unsplit(plan):
    # config 2: 3x3 s1 p1, batch 32, 64 -> 64 channels, 32x32: 32768 rows, 9 taps x 4 steps of 16 channels
    kernel, rows, ksplit, steps, wgs = plan(1, 8, 0, 64, 64, 3, 3, 1, 32 * 32 * 32, 32, 1)
    assert (kernel, rows, ksplit, steps, wgs) == (QUAD, 1024, 1, 36, 256)


def test_resnet20_layers(plan):
    # first layer: 3 channels (padded to 8): no quad tables; x-major copy, 128-byte lines, paired taps
    assert plan(1, 8, 0, 16, 3, 3, 3, 1, 128 * 32 * 32, 32, 1)[:3] == (XMAJOR, 1024, 1)
    # stage 1: 16 channels, 9 steps of 16, 131072 rows x 2 channel tiles: quad kernel, 4 rows per row slot, 256 workgroups
    assert plan(1, 8, 0, 16, 16, 3, 3, 1, 128 * 32 * 32, 32, 1) == (QUAD, 1024, 1, 9, 256)
    # a 1x1 layer of 32 channels has 2 steps: below the quad kernel's minimum of 4
    assert plan(1, 8, 0, 16, 32, 1, 1, 1, 128 * 32 * 32, 32, 1)[0] != QUAD
    # stage 2: 32 channels, 32768 rows: unsplit the quad kernel would cover half the compute units: 2 slices of 9 steps
    assert plan(1, 8, 0, 32, 32, 3, 3, 1, 128 * 16 * 16, 16, 1) == (QUAD, 1024, 2, 18, 256)
    # stage 3: 64 channels, 8192 rows: a quarter of the compute units: 4 slices of 9 steps
    assert plan(1, 8, 0, 64, 64, 3, 3, 1, 128 * 8 * 8, 8, 1) == (QUAD, 1024, 4, 36, 256)
    # too few steps to slice (a 1x1 layer of 64 channels, 4 steps, on a quarter of the chip): 128-byte-line kernels
    assert plan(1, 8, 0, 64, 64, 1, 1, 1, 128 * 8 * 8, 8, 1)[0] != QUAD
    # stride-2 layers never take the x-major copy
    assert plan(1, 8, 0, 32, 16, 3, 3, 1, 128 * 16 * 16, 16, 2)[0] in (FAST, GENERIC)
    assert plan(1, 8, 0, 64, 32, 3, 3, 1, 128 * 8 * 8, 8, 2)[0] in (FAST, GENERIC)
    # final linear layer, 128 rows: whole-table kernel
    assert plan(0, 8, 0, 10, 64, 1, 1, 1, 128, 128, 1)[0] == ROWS


def test_lstm_layers(plan):
    # input products of all time steps: 6400 rows x 512 -> 2048, 7-bit table: quad kernel, 2048 rows per workgroup
    k, rows, ksplit, steps, wgs = plan(0, 7, 0, 2048, 512, 1, 1, 1, 100 * 64, 100 * 64, 1)
    assert (k, rows, ksplit, steps) == (QUAD, 2048, 1, 32) and wgs == 4 * 256
    # one time step of the recurrence: 64 rows: whole-table kernel
    assert plan(0, 7, 0, 2048, 512, 1, 1, 1, 64, 64, 1)[0] == ROWS


@pytest.mark.parametrize("bits", [6, 8])
def test_generator_layers(plan, bits):
    # stride-2 4x4 transposed convolutions = 4 phases of 2x2 taps; rows per phase = batch x input pixels
    for cin, cout, hw in ((512, 256, 4), (256, 128, 8), (128, 64, 16), (64, 3, 32)):
        k, rows, ksplit, steps, wgs = plan(2, bits, 0, cout, cin, 4, 4, 2, 256 * hw * hw, hw, 1)
        assert (k, rows, ksplit, steps) == (QUAD, 2048, 1, 4 * cin // 16), (cin, cout)
        assert wgs == (256 * hw * hw // 2048) * ((cout + 7) // 8) * 4


def test_two_pass_tables_stay_off_the_quad_kernel(plan):
    assert plan(1, 8, 1, 64, 64, 3, 3, 1, 32 * 32 * 32, 32, 1)[0] != QUAD


def test_bad_arguments(plan):
    from paper_2203_04071_amd import binding as B
    with pytest.raises(B.AdaptError):
        plan(3, 8, 0, 64, 64, 3, 3, 1, 1024, 32, 1)
    with pytest.raises(B.AdaptError):
        plan(1, 9, 0, 64, 64, 3, 3, 1, 1024, 32, 1)
