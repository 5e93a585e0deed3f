"""Host logic of gp_lc_forward: arguments are validated before anything touches a
GPU, so the error paths run without one."""
import pytest

import paper_2207_12000_amd as gp


def call(**kw):
    a = dict(stack_ptr=4096, ld=8, dtype=gp.GP_F32, n=10, d=8, K=1, batch_ptr=None, B=4, gamma=[1.0, 1.0],
             weight_ptrs=[4096], widths=[4], out_ptr=4096, ldo=4)
    a.update(kw)
    gp.gp_lc_forward(**a)


@pytest.mark.parametrize("kw,status", [
    (dict(stack_ptr=0), gp.GP_ERR_INVALID_ARG),
    (dict(out_ptr=0), gp.GP_ERR_INVALID_ARG),
    (dict(weight_ptrs=[0]), gp.GP_ERR_INVALID_ARG),
    (dict(dtype=5), gp.GP_ERR_INVALID_ARG),
    (dict(ld=7), gp.GP_ERR_INVALID_ARG),
    (dict(n=0), gp.GP_ERR_INVALID_ARG),
    (dict(d=0, ld=0), gp.GP_ERR_INVALID_ARG),
    (dict(B=-1), gp.GP_ERR_INVALID_ARG),
    (dict(B=11), gp.GP_ERR_INVALID_ARG),                       # no batch list: rows 0 .. B-1 must exist
    (dict(ldo=3), gp.GP_ERR_INVALID_ARG),
    (dict(K=16, gamma=[0.0] * 17), gp.GP_ERR_UNSUPPORTED),
    (dict(weight_ptrs=[], widths=[]), gp.GP_ERR_UNSUPPORTED),
    (dict(weight_ptrs=[4096] * 9, widths=[4] * 9), gp.GP_ERR_UNSUPPORTED),
    (dict(widths=[257], ldo=257), gp.GP_ERR_UNSUPPORTED),
    (dict(widths=[0]), gp.GP_ERR_UNSUPPORTED),
])
def test_rejected_arguments(kw, status):
    with pytest.raises(gp.GpError) as e:
        call(**kw)
    assert e.value.status == status
    assert gp.gp_last_error()


def test_empty_batch_is_a_no_op():
    call(B=0)                                                   # returns before any device work


def test_gamma_length_is_checked_by_the_binding():
    with pytest.raises(ValueError):
        call(gamma=[1.0])


def call_branches(**kw):
    a = dict(stack_ptr=4096, ld=8, dtype=gp.GP_F32, n=10, d=8, K=2, batch_ptr=None, B=4, gamma=[1.0, 1.0, 1.0],
             depth=[0, 1, 2], comb=gp.GP_COMB_CONCAT, weight_ptrs=[4096, 4096], widths=[4, 6], out_ptr=4096, ldo=10)
    a.update(kw)
    gp.gp_lc_forward_branches(**a)


@pytest.mark.parametrize("kw,status", [
    (dict(depth=[0, 0, 0]), gp.GP_ERR_INVALID_ARG),                       # every hop left out
    (dict(depth=[0, 1, 3]), gp.GP_ERR_INVALID_ARG),                       # deeper than the weight list
    (dict(depth=[0, -1, 2]), gp.GP_ERR_INVALID_ARG),
    (dict(comb=3), gp.GP_ERR_INVALID_ARG),
    (dict(comb=gp.GP_COMB_SUM), gp.GP_ERR_INVALID_ARG),                   # widths 4 and 6 cannot be summed
    (dict(comb=gp.GP_COMB_MAX), gp.GP_ERR_INVALID_ARG),
    (dict(ldo=9), gp.GP_ERR_INVALID_ARG),                                 # concatenation is 4 + 6 columns wide
])
def test_branches_rejected_arguments(kw, status):
    with pytest.raises(gp.GpError) as e:
        call_branches(**kw)
    assert e.value.status == status


def test_branches_empty_batch_is_a_no_op():
    call_branches(B=0)
    call_branches(B=0, comb=gp.GP_COMB_MAX, widths=[6, 6], ldo=6)


@pytest.mark.parametrize("args", [(0, 4, 4, 4), (4096, -1, 4, 4), (4096, 4, 0, 4), (4096, 4, 5, 4)])
def test_softmax_rejected_arguments(args):
    with pytest.raises(gp.GpError) as e:
        gp.gp_lc_softmax(*args)
    assert e.value.status == gp.GP_ERR_INVALID_ARG


def test_softmax_of_no_rows_is_a_no_op():
    gp.gp_lc_softmax(4096, 0, 4, 4)
