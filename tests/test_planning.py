"""Host-side planning helpers: sync schedules and the analytic cost report (no GPU)."""
import numpy as np
import pytest

from oracle import rowwise as oracle
from paper_2511_02647_amd.planning import cost_report, sync_schedule, uniform_schedule

NAMES = ("uniform", "shallow-half", "deep-half", "progressive", "regressive")


@pytest.mark.parametrize("M,H", [(8, 1), (8, 4), (32, 4), (5, 2), (7, 7), (6, 0), (6, -1), (4, 9)])
def test_uniform_schedule_is_algorithm_1(M, H):
    # Algorithm 1: with m = H t + h, the block with h = H runs global attention
    flags = uniform_schedule(M, H)
    assert flags == [oracle.is_sync_block(H, b) for b in range(M)]
    assert sum(flags) == (M // H if H >= 1 else 0)


@pytest.mark.parametrize("M,T", [(8, 4), (32, 8), (32, 1), (5, 5), (28, 7), (9, 0), (33, 6)])
def test_schedule_presets_place_the_budget(M, T):
    for name in NAMES:
        flags = sync_schedule(name, M, T)
        assert len(flags) == M and sum(flags) == T, name
    if T == 0:
        return
    idx = {name: [i for i, f in enumerate(sync_schedule(name, M, T)) if f] for name in NAMES}
    half = max(T, M // 2)
    assert all(i < half for i in idx["shallow-half"])
    assert all(i >= M - half for i in idx["deep-half"])
    gaps = lambda ix: [ix[0] + 1] + [b - a for a, b in zip(ix, ix[1:])]
    gp, gr = gaps(idx["progressive"]), gaps(idx["regressive"])
    assert gp == sorted(gp) and gr == sorted(gr, reverse=True)      # intervals grow / shrink with depth
    assert gr == gp[::-1]
    for name in ("uniform", "progressive", "regressive", "deep-half"):
        assert idx[name][-1] == M - 1, name                        # the stack ends on a global block
    if M % T == 0:
        assert sync_schedule("uniform", M, T) == uniform_schedule(M, M // T)


def test_schedule_rejects_bad_budget():
    with pytest.raises(ValueError):
        sync_schedule("uniform", 4, 5)
    with pytest.raises(ValueError):
        sync_schedule("nonsense", 4, 2)


def test_cost_report_closed_forms():
    # equal segments, dense exchange: every global block a participant sends L rows of K and V
    # and receives (N - 1) L
    N, L, Hq, Hkv, D, M, H = 4, 512, 32, 8, 128, 32, 4
    flags = uniform_schedule(M, H)
    r = cost_report([L] * N, flags, Hq, Hkv, D)
    row_bits = 2 * Hkv * D * 2 * 8
    assert r.n_sync_blocks == 8
    assert r.comm_bits_sent_per_participant == 8 * L * row_bits
    assert r.comm_bits_per_participant == 8 * N * L * row_bits
    # FLOPs: summed over participants = 4 D Hq (pairs of a block-diagonal causal mask in local
    # blocks, of the full causal mask in global blocks)
    local_pairs = N * L * (L + 1) // 2
    sync_pairs = (N * L) * (N * L + 1) // 2
    assert r.prefill_attn_flops_per_participant * N == 4 * D * Hq * (24 * local_pairs + 8 * sync_pairs)
    # memory: own K, V in local blocks, the global K, V in global blocks
    assert r.peak_kv_bytes_per_participant == (24 * L + 8 * N * L) * 2 * Hkv * D * 2


def test_cost_report_sparse_and_never_sync():
    lens = [100, 300, 50]
    none = cost_report(lens, [False] * 6, 8, 2, 64)
    assert none.comm_bits_per_participant == 0 and none.n_sync_blocks == 0
    dense = cost_report(lens, [True] * 6, 8, 2, 64)
    quarter = cost_report(lens, [True] * 6, 8, 2, 64, keep_fraction=0.25)
    assert quarter.comm_bits_per_participant < 0.3 * dense.comm_bits_per_participant
    # own rows stay complete under sparse exchange: the cost never drops below the local one
    assert quarter.prefill_attn_flops_per_participant > none.prefill_attn_flops_per_participant
    # brute force of the visible-pair count behind the FLOPs, dense exchange
    seg = np.concatenate([[0], np.cumsum(lens)])
    pairs = 0
    for i in range(seg[-1]):
        pairs += i + 1
    assert dense.prefill_attn_flops_per_participant * 3 == 4 * 64 * 8 * 6 * pairs
