"""Host logic of the multi-layer call (no GPU): which layers sqllm_dense_sparse_matvec_multi launches together and with how many
rows per workgroup, through sqllm_multi_launch_order.  Expected values are worked out by hand from the rule the header states:
a group is (plan or no plan, waves per workgroup, and without a plan the row class of the layer's own launch); groups in the
order of their first layer; up to 16 planned or 8 unplanned layers per launch; planned launches of several layers take eight
rows from 4096 eight-row workgroups on, or when their rows have 16384 columns or more."""
import numpy as np
import pytest

import paper_2306_07629_amd as sq
from paper_2306_07629_amd import binding

A = 0x7F0000001000          # a plausible, well-aligned address: the call follows no pointer


def layer(M, N, nnz=5, plan=False, bits=3):
    return (M, N, bits, nnz, A, A, A, A, A, A, A) + ((A,) if plan else ())


def test_one_decoder_block_with_plans_is_two_launches():
    block = [layer(4096, 4096, plan=True)] * 4 + [layer(11008, 4096, plan=True)] * 2 + [layer(4096, 11008, plan=True)]
    launch, rows, n = sq.sqllm_multi_launch_order(block)
    assert launch == [0, 0, 0, 0, 0, 0, 1] and n == 2
    # 4 x 512 + 2 x 1376 = 4800 eight-row workgroups: eight rows; the lonely 11008-wide layer is its own launch (six waves, rule 4)
    assert rows == [8] * 6 + [4]


def test_a_whole_step_is_twelve_plus_two_launches_of_sixteen():
    block = [layer(4096, 4096, plan=True)] * 4 + [layer(11008, 4096, plan=True)] * 2 + [layer(4096, 11008, plan=True)]
    launch, rows, n = sq.sqllm_multi_launch_order(block * 32)
    assert n == 14 and set(rows) == {8}
    narrow = [launch[i] for i in range(224) if i % 7 != 6]
    wide = [launch[i] for i in range(224) if i % 7 == 6]
    assert narrow == sorted(narrow) and narrow == [k // 16 for k in range(192)]      # launches 0 .. 11 in layer order
    assert wide == [12] * 16 + [13] * 16


def test_without_a_plan_a_launch_holds_eight_layers_and_keeps_the_layers_own_rows():
    block = [layer(4096, 4096)] * 4 + [layer(11008, 4096)] * 2 + [layer(4096, 11008)]
    launch, rows, n = sq.sqllm_multi_launch_order(block * 32)
    assert n == 24 + 4 and set(rows) == {4}
    wide = [layer(64, 16384)] * 3 + [layer(64, 4096)] + [layer(64, 16384)]
    launch, rows, n = sq.sqllm_multi_launch_order(wide)
    assert launch == [0, 0, 0, 1, 0] and rows == [8, 8, 8, 4, 8] and n == 2


def test_groups_of_projections_that_share_an_input():
    q = layer(4096, 4096, plan=True)
    launch, rows, n = sq.sqllm_multi_launch_order([q, q, q])
    assert launch == [0, 0, 0] and rows == [4, 4, 4] and n == 1                    # 1536 eight-row workgroups: four rows
    launch, rows, n = sq.sqllm_multi_launch_order([layer(11008, 4096, plan=True)] * 2)
    assert rows == [4, 4] and n == 1                                               # 2752
    launch, rows, n = sq.sqllm_multi_launch_order([layer(11008, 4096, plan=True)] * 3)
    assert rows == [8, 8, 8] and n == 1                                            # 4128 >= 4096


def test_plan_and_no_plan_and_empty_layers_and_layers_without_nonzeros():
    ls = [layer(8, 4096, plan=True), layer(8, 4096), layer(0, 4096, plan=True), layer(8, 4096, nnz=0, plan=True), layer(8, 4096, plan=True),
          layer(8, 4096, nnz=0), layer(8, 2048), layer(8, 4096)]
    launch, rows, n = sq.sqllm_multi_launch_order(ls)
    # layer 3 has a plan pointer but no nonzeros: it is an unplanned layer of two waves (no sparse wave), like layer 5;
    # layers 1 and 7 are unplanned with a sparse wave (three waves); layer 6 has one dense wave and the sparse wave (two waves, as 3 and 5)
    assert launch == [0, 1, -1, 2, 0, 2, 2, 1] and n == 3
    assert rows == [4, 4, 0, 4, 4, 4, 4, 4]


def test_seventeen_planned_layers_split_sixteen_and_one():
    launch, rows, n = sq.sqllm_multi_launch_order([layer(16, 2048, plan=True)] * 17)
    assert launch == [0] * 16 + [1] and n == 2


def test_against_a_restatement_of_the_rule_on_random_calls():
    rng = np.random.default_rng(5)
    for trial in range(50):
        count = int(rng.integers(1, 400))
        ls, want_key = [], []
        for _ in range(count):
            M = int(rng.choice([0, 1, 7, 512, 4096, 11008, 40000]))
            N = int(rng.choice([128, 2048, 2176, 4096, 11008, 16384, 22016, 28672]))
            nnz = int(rng.choice([0, 9]))
            plan = bool(rng.integers(0, 2))
            ls.append(layer(M, N, nnz=nnz, plan=plan))
            planned = plan and nnz > 0
            W = -(-N // 2048)
            want_key.append(None if M == 0 else (planned, W + (0 if planned or nnz == 0 else 1), None if planned else (8 if W >= 8 else 4)))
        launch, rows, n = sq.sqllm_multi_launch_order(ls)
        # walk the rule: groups in order of first appearance, chunks of 16 / 8 in layer order
        expect, rows_expect, k = [-1] * count, [0] * count, 0
        seen = []
        for key in want_key:
            if key is not None and key not in seen:
                seen.append(key)
        for key in seen:
            members = [i for i in range(count) if want_key[i] == key]
            cap = 16 if key[0] else 8
            for c in range(0, len(members), cap):
                chunk = members[c:c + cap]
                blocks8 = sum(-(-ls[i][0] // 8) for i in chunk)
                W = -(-ls[chunk[0]][1] // 2048)
                r = (8 if (W >= 8 or (len(chunk) > 1 and blocks8 >= 4096)) else 4) if key[0] else key[2]
                for i in chunk:
                    expect[i], rows_expect[i] = k, r
                k += 1
        assert launch == expect and rows == rows_expect and n == k, trial


def test_errors():
    with pytest.raises(sq.SqllmError) as e:
        sq.sqllm_multi_launch_order([layer(4, 128), layer(4, 100)])
    assert binding.STATUS_NAMES[e.value.status] == "SQLLM_ERR_SHAPE" and "layer 1" in str(e.value)
    L = sq.lib()
    arr = sq.layer_descriptors([layer(4, 128)])
    assert L.sqllm_multi_launch_order(1, arr, None, None, None) == binding.STATUS_NAMES.index("SQLLM_ERR_NULL")
    assert L.sqllm_multi_launch_order(0, None, None, None, None) == 0
    assert sq.sqllm_multi_launch_order([]) == ([], [], 0)
