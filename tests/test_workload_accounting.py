"""The algorithmic byte count that the roofline figure of bench.py divides by the launch time,
checked against a count made unit by unit, token by token."""
from paper_2404_04793_amd import workloads as W


def _count_by_hand(wl, budgets, t):
    row = wl.D * wl.elem_bytes
    total = 0
    for b in budgets:
        for _unit in range(wl.B * wl.Hkv):
            kept = min(wl.P + t + 1, b)
            for _tok in range(kept):
                total += row + row                      # its K row and its V row, read once
                if wl.policy == "h2o":
                    total += 4 + 4                      # accumulated score: read, write
            total += row + row                          # the appended token's K and V rows, written
        total += wl.B * wl.Hq * wl.D * wl.elem_bytes    # q read
        total += wl.B * wl.Hq * wl.D * wl.elem_bytes    # out written
    return total


def test_tiny_counts_match_a_token_by_token_count():
    wl = W.WORKLOADS["tiny"]
    budgets = [85, 17, 17, 85]
    got = W.decode_bytes_per_step(wl, budgets)
    assert len(got) == wl.S
    for t in (0, 7, wl.S - 1):
        assert got[t] == _count_by_hand(wl, budgets, t)
    streaming = W.scaled(wl, policy="streaming")
    assert W.decode_bytes_per_step(streaming, budgets)[3] == _count_by_hand(streaming, budgets, 3)


def test_llama2_7b_mean_is_the_figure_of_the_profile():
    wl = W.WORKLOADS["llama2_7b"]
    budgets = [2271, 2271] + [143] * 28 + [2271, 2271]
    per_step = W.decode_bytes_per_step(wl, budgets)
    assert sum(per_step) // wl.S == 1699176928
    # 512 bytes of K and V plus 8 bytes of score per kept token and KV head, the dominant term
    full = 256 * (28 * 143 + 4 * 2271) * 520
    assert 0.99 < full / per_step[-1] < 1.0


def test_ragged_count_reduces_to_the_uniform_one_and_counts_each_sequence():
    wl = W.scaled(W.WORKLOADS["tiny"], B=3)
    budgets = [85, 17, 17, 85]
    same = W.decode_bytes_per_step_ragged(wl, [[b] * 3 for b in budgets], [wl.P] * 3)
    assert same == W.decode_bytes_per_step(wl, budgets)
    # one sequence with a shorter prompt and smaller budgets: only its own units change
    one = W.scaled(wl, B=1)
    a = W.decode_bytes_per_step(one, budgets)
    b = W.decode_bytes_per_step_ragged(W.scaled(one, P=100), [[40], [9], [9], [40]], [100])
    mixed = W.decode_bytes_per_step_ragged(wl, [[85, 40, 85], [17, 9, 17], [17, 9, 17], [85, 40, 85]], [wl.P, 100, wl.P])
    assert [x - 2 * y for x, y in zip(mixed, a)] == b


def test_kv_size_model_is_the_papers():
    """Sec. 2.1: Llama-2-7B in 16 bits caches 2 * 32 * 4096 * 2 bytes = 0.5 MB per token; a KV head layout
    with fewer heads shrinks it by the group size."""
    assert W.kv_bytes_per_token(W.WORKLOADS["llama2_7b"]) == 2 * 32 * 4096 * 2 == 512 * 1024
    assert W.kv_bytes_per_token(W.WORKLOADS["mistral_7b"]) == 512 * 1024 // 4
    assert W.kv_bytes_per_token(W.WORKLOADS["llama2_70b"]) == 2 * 80 * 8 * 128 * 2
    stress = W.WORKLOADS["stress_7b"]
    assert W.full_cache_bytes_per_sequence(stress) == 1536 * 512 * 1024          # 805 MB for 512 + 1024 tokens


def test_resident_bytes_and_the_equal_memory_batch_of_the_stress_configuration():
    """Budgets 35 x 28 layers + 571 x 4 layers (20 % of a 512-token prompt, p = 0.35): 3264 slots per
    sequence and KV head, 520 bytes each under H2O -> 12.17 GB at batch 224; an uncompressed cache for the
    whole 1536-token generation needs 805 MB per sequence, so 15 sequences fit in the same memory."""
    stress = W.WORKLOADS["stress_7b"]
    budgets = [571, 571] + [35] * 28 + [571, 571]
    assert sum(budgets) == stress.total_budget == 3264
    squeezed = W.squeezed_cache_bytes(stress, budgets)
    assert squeezed == 224 * 32 * 3264 * (2 * 128 * 2 + 8)
    assert W.resident_cache_bytes(stress, [224 * 32 * b for b in budgets]) == squeezed
    assert W.equal_memory_batch(stress, squeezed) == 15
    # a budget above what a sequence can ever hold only costs the slots that can fill
    short = W.scaled(stress, S=8)
    assert W.squeezed_cache_bytes(short, [571]) == 224 * 32 * 520 * 520
    # without an accumulator (sliding window, StreamingLLM) a slot carries its rows and its position
    assert W.resident_cache_bytes(W.WORKLOADS["llama2_70b"], [10]) == 10 * (512 + 4)
    # the uncompressed cache of the whole batch, for scale: 224 x 805 MB = 180 GB
    assert 224 * W.full_cache_bytes_per_sequence(stress) == 180388626432
