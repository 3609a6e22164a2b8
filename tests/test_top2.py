"""Greedy sampling with a confidence gap (Sec. 3.8, Sec. 3.9.2, Sec. 3.9.4): pins for the oracle
(CPU) and parity of the HIP path (GPU).  Everything is a selection among the given fp32 values,
so indices and values are compared exactly."""
import numpy as np
import pytest
import torch

import oracle
import paper_2605_13784_amd as sk
from workloads import synth


def _brute(row):
    """Pure-Python scan: best and second best by (value descending, index ascending)."""
    order = sorted(range(len(row)), key=lambda i: (-float(row[i]), i))
    return order[0], order[1]


def test_oracle_against_brute_force_and_ties():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 13)).astype(np.float32)
    x[1, 4] = x[1, 9] = x[1].max() + 1.0                 # two equal maxima: lower index first, gap 0
    x[2, :] = 0.5                                        # all equal: indices 0 and 1
    x[3, 0] = 5.0; x[3, 1:] = -np.inf                    # a single finite entry
    x[4, 12] = 9.0; x[4, 11] = 8.0                       # maximum in the last place
    x[5] = np.arange(13, dtype=np.float32)               # increasing: last, last but one
    x[6] = -np.arange(13, dtype=np.float32)              # decreasing: 0, 1
    i1, i2, v1, v2, gap = oracle.top2(x)
    for r in range(7):
        b1, b2 = _brute(x[r])
        assert (i1[r], i2[r]) == (b1, b2)
        assert v1[r] == x[r, b1] and v2[r] == x[r, b2]
    assert (i1[1], i2[1], gap[1]) == (4, 9, 0.0)
    assert (i1[2], i2[2]) == (0, 1) and (i1[3], i2[3]) == (0, 1) and gap[3] == np.inf
    assert (i1[5], i2[5], gap[5]) == (12, 11, 1.0) and (i1[6], i2[6]) == (0, 1)
    assert np.all(gap >= 0)
    # permuting a row moves the indices with the values
    perm = rng.permutation(13)
    j1, j2, w1, w2, _ = oracle.top2(x[0:1, perm])
    assert perm[j1[0]] == i1[0] and perm[j2[0]] == i2[0] and w1[0] == v1[0] and w2[0] == v2[0]
    with pytest.raises(ValueError):
        oracle.top2(np.zeros((2, 1), np.float32))


def test_library_rejects_bad_arguments_without_a_gpu():
    lib = sk.lib()
    assert lib.sk_top2_workspace_bytes(0, 100) == 0 and lib.sk_top2_workspace_bytes(4, 1) == 0
    assert lib.sk_top2_workspace_bytes(64, 128256) == 64 * 16 * 16
    assert lib.sk_top2(None, 3, 1, 1, None, 0, None, None, None, None, None, None) == sk.SK_E_INVAL
    assert lib.sk_top2(None, 0, 100, 100, None, 0, None, None, None, None, None, None) == sk.SK_OK


@pytest.mark.gpu
@pytest.mark.parametrize("rows,vocab,stride", [(1, 128256, 128256), (64, 128256, 128256), (5, 2, 4), (3, 8191, 8192),
                                               (7, 8193, 8196), (2, 32000, 40000), (130, 50257, 50260)])
def test_gpu_top2_equals_oracle_exactly(rows, vocab, stride):
    """Synthetic logits N(0, 2.5) in the shapes of a 128k-vocabulary model (and ragged ones that end
    inside a float4, inside and just behind a workgroup's chunk), planted ties included."""
    gen = synth.generator(6, stream=rows + vocab)
    buf = 2.5 * synth.draw(gen, (rows, stride), "f32")
    x = buf[:, :vocab]
    buf[:, vocab:] = 1e30                                 # what lies behind the row must not count
    if vocab > 16:
        x[0, vocab - 1] = x[0].max() + 1.0                # maximum in the last place
        if rows > 1:
            x[1, 7] = x[1, vocab // 2] = x[1].max() + 2.0    # equal maxima, chunks apart
        if rows > 2:
            x[2, :] = -1.0                                # all equal
        if rows > 3:
            x[3, :] = -np.inf; x[3, 5] = 1.0              # one finite entry: runner-up is the lowest other index
        if rows > 4:
            x[4, :] = -np.inf                             # nothing finite at all: indices 0 and 1
    xd = buf.cuda()[:, :vocab]
    i1, i2, v1, v2, gap = sk.sk_top2(xd)
    torch.cuda.synchronize()
    r1, r2, w1, w2, g = oracle.top2(x.numpy())
    np.testing.assert_array_equal(i1.cpu().numpy(), r1)
    np.testing.assert_array_equal(i2.cpu().numpy(), r2)
    np.testing.assert_array_equal(v1.cpu().numpy(), w1)
    np.testing.assert_array_equal(v2.cpu().numpy(), w2)
    np.testing.assert_array_equal(gap.cpu().numpy(), g)


@pytest.mark.gpu
def test_gpu_top2_workspace_too_small_is_an_error():
    x = torch.zeros((4, 20000), dtype=torch.float32, device="cuda")
    with pytest.raises(sk.SkError) as e:
        sk.sk_top2(x, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == sk.SK_E_WORKSPACE
