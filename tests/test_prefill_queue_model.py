"""The ticket -> item mapping of the matrix-core prefill kernel's work queues, restated on the host and
checked exhaustively: with any shares, every item of the batch is handed out exactly once.

The kernel (csrc/attn_prefill_mfma.hip: the quota block and resolve()) deals item f to queue f % 8; a queue
whose XCD was slow in the launch before works through fewer items than its own list holds, and the ends of
such lists are dealt, in queue order, to the queues that take more than their own.  This file holds the same
arithmetic in plain Python; the GPU test test_config3_prefill_queue_shares_follow_the_xcds_and_change_no_result
checks the kernel itself (bit-identical outputs whatever the shares)."""
import numpy as np
import pytest

Q = 8
MIN_ITEMS = 3072


def quotas(n_flat, grid, share):
    big = n_flat >= MIN_ITEMS and grid <= 1024 and grid % Q == 0
    own = [max(n_flat - x + Q - 1, 0) // Q for x in range(Q)]
    crew = [(grid - x + Q - 1) // Q for x in range(Q)]
    sh = np.asarray(share, dtype=np.float32)
    sh = sh * np.float32(8.0) / np.float32(sh.sum())
    quota = [int(np.float32(own[x]) * sh[x] + np.float32(0.5)) for x in range(Q)]
    quota[Q - 1] += n_flat - sum(quota)
    ok = big and all(quota[x] >= 2 * crew[x] and own[x] >= 2 * crew[x] for x in range(Q))
    return (quota if ok else list(own)), own, ok


def resolve(k, q, quota, own):
    if k < min(quota[q], own[q]):
        return Q * k + q
    if k >= quota[q]:
        return -1
    p = k - own[q]
    for x in range(q):
        p += max(quota[x] - own[x], 0)
    for d in range(Q):
        cnt = own[d] - quota[d]
        if cnt <= 0:
            continue
        if p < cnt:
            return Q * (quota[d] + p) + d
        p -= cnt
    return -1


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_every_item_is_handed_out_exactly_once(seed):
    rng = np.random.default_rng(seed)
    balanced = 0
    for _ in range(150):
        n_flat = int(rng.integers(2000, 30000))
        grid = int(rng.choice([512, 256, 1024, 608]))
        share = np.clip(rng.normal(1.0, 0.25, Q), 0.5, 1.5)
        quota, own, ok = quotas(n_flat, grid, share)
        balanced += ok
        assert sum(quota) == n_flat == sum(own)
        seen = np.zeros(n_flat, np.int32)
        for q in range(Q):
            k = 0
            while True:
                f = resolve(k, q, quota, own)
                if f < 0:
                    break
                seen[f] += 1
                k += 1
            assert k == quota[q]
            assert resolve(k + 3, q, quota, own) == -1
            # the first two rounds of a queue's crew (fixed tickets) come from its own list
            crew = (grid - q + Q - 1) // Q
            assert all(resolve(j, q, quota, own) == Q * j + q for j in range(min(2 * crew, own[q], quota[q])))
        assert (seen == 1).all()
    assert balanced > 50


def test_what_changes_hands_is_the_light_end_of_a_list():
    quota, own, ok = quotas(8000, 512, [0.8, 1.2, 1.0, 1.0, 0.9, 1.1, 1.0, 1.0])
    assert ok
    # queue 0 gives away the last 200 of its 1000 items; queue 1, the first taker, gets them in order
    assert own[0] == 1000 and quota[0] == 800 and quota[1] == 1200
    assert resolve(799, 0, quota, own) == Q * 799 and resolve(800, 0, quota, own) == -1
    assert resolve(1000, 1, quota, own) == Q * 800 + 0 and resolve(1199, 1, quota, own) == Q * 999 + 0
    # queue 4 gives 100 away, which go to queue 5 (the second taker)
    assert resolve(1000, 5, quota, own) == Q * 900 + 4
