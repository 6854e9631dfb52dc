"""The comparator behind the every-element GPU tests, checked on the CPU: it must report
zero for the oracle's own result and count every planted difference, in every array, at
both ends of every thread's range."""
import numpy as np

from oracle import step as orc
from synth import host as gen

from gpu_util import oracle_mismatches


def _case(n=40_003, N=4, t=7):
    grads = [gen.gradient(n, 5, 0, r, "bf16", 1e-3) for r in range(N)]
    pre = [gen.master(n, 5), *gen.moments(n, 5, True)]
    s = orc.derive_scalars(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, t=t, n_devices=N)
    post = [a.copy() for a in pre] + [np.zeros(n, np.uint16)]
    orc.step_f32(grads, s, *post)
    return grads, pre, s, post


def test_oracle_result_has_no_mismatch_and_planted_ones_are_counted():
    grads, pre, s, post = _case()
    n = pre[0].shape[0]
    assert oracle_mismatches(orc.step_f32, s, grads, [a.copy() for a in pre], post, n) == [0, 0, 0, 0]
    # one flipped low bit per array, at the first element, the last, and inside
    for j in range(4):
        for e in (0, n - 1, n // 3):
            bad = [a.copy() for a in post]
            bits = bad[j].view(np.uint16 if j == 3 else np.uint32)
            bits[e] ^= 1
            want = [0, 0, 0, 0]
            want[j] = 1
            assert oracle_mismatches(orc.step_f32, s, grads, [a.copy() for a in pre], bad, n) == want
    # only [0, count) is compared
    bad = [a.copy() for a in post]
    bad[0].view(np.uint32)[n - 1] ^= 1
    assert oracle_mismatches(orc.step_f32, s, grads, [a.copy() for a in pre], bad, n - 1) == [0, 0, 0, 0]


def test_a_wrong_contribution_or_a_stale_state_is_noticed_everywhere():
    grads, pre, s, post = _case()
    n = pre[0].shape[0]
    swapped = [grads[0], grads[1], grads[1], grads[3]]            # a wrong pointer for contribution 2
    got = oracle_mismatches(orc.step_f32, s, swapped, [a.copy() for a in pre], post, n)
    assert min(got[:3]) > 0.9 * n                                 # nearly every element of master, m, v
    stale = [pre[0].copy(), post[1].copy(), post[2].copy(), post[3].copy()]   # master not updated
    got = oracle_mismatches(orc.step_f32, s, grads, [a.copy() for a in pre], stale, n)
    assert got[0] > 0.9 * n and got[1] == 0 and got[2] == 0 and got[3] == 0
    for threads in (1, 3, 16, 64):                                 # any split of the range gives the same counts
        assert oracle_mismatches(orc.step_f32, s, grads, [a.copy() for a in pre], post, n, threads) == [0, 0, 0, 0]
