"""Approximation-schedule masks against the counts the paper prints (Sections 3, 3.4)."""
import numpy as np

from paper_1908_05460_amd import inputs, schedule as sch


def test_schedule1_layer_counts_printed_in_the_paper():
    vgg, res = len(inputs.vgg19_stack()), len(inputs.resnet20_stack())
    assert (vgg, res) == (16, 19)
    assert np.flatnonzero(sch.schedule1(vgg, 0)).tolist() == [1, 5, 9, 13]       # layers 2,6,10,14
    assert np.flatnonzero(sch.schedule1(res, 7)).tolist() == [1, 5, 9, 13, 17]   # five layers
    assert sch.schedule1(res, 0)[0] == sch.EXACT                                  # first conv untouched


def test_all_three_paper_schedules_target_a_quarter():
    for fn in sch.PAPER_SCHEDULES.values():
        assert abs(sch.fraction_approximated(fn, 19, 400) - 0.25) < 0.03
        assert abs(sch.fraction_approximated(fn, 16, 400) - 0.25) < 0.01


def test_sweep_masks():
    n = 19
    assert not sch.all_exact(n, 3).any()
    assert np.flatnonzero(sch.every_other_layer(n, 0)).tolist() == list(range(1, 19, 2))
    m = sch.all_but_first_and_last(n, 0)
    assert m[0] == sch.EXACT and m[-1] == sch.EXACT and (m[1:-1] == sch.APPROX).all()
    assert not sch.alternate_batches(n, 0).any() and (sch.alternate_batches(n, 1) == sch.APPROX).all()
    assert (sch.schedule1(n, 0, sch.ZERO)[[1, 5]] == sch.ZERO).all()


def test_layer_tables_match_the_stated_stacks():
    res = inputs.resnet20_stack()
    assert [(l.C, l.K, l.H, l.stride) for l in res[:2]] == [(3, 16, 32, 1), (16, 16, 32, 1)]
    assert (res[7].C, res[7].K, res[7].H, res[7].stride, res[7].Ho) == (16, 32, 32, 2, 16)
    assert (res[13].C, res[13].K, res[13].H, res[13].stride, res[13].Ho) == (32, 64, 16, 2, 8)
    assert all(l.H == 8 and l.C == 64 for l in res[14:])
    vgg = inputs.vgg19_stack()
    assert [l.H for l in vgg] == [32, 32, 16, 16, 8, 8, 8, 8, 4, 4, 4, 4, 2, 2, 2, 2]
    assert abs(sum(l.flops(128) for l in res) / 1e9 - 10.38) < 0.01              # nominal GFLOP
    assert abs(sum(l.flops(128) for l in vgg) / 1e9 - 101.9) < 0.1
