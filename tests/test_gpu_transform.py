"""GPU dense transform (fp32 matrix cores) against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_13053_amd import binding as B
from paper_2302_13053_amd import harness as Hn
from paper_2302_13053_amd import workloads as wl
from parity import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(autouse=True)
def kernel_family(transform_family):
    """Every test of this file runs on both kernel families."""
    return transform_family


def run(n, d_in, d_out, ldh, ldz, relu, bias, seed):
    H = wl.random_matrix(n, d_in, seed, ld=ldh)
    H[:, d_in:] = np.nan                                   # padding must never be read into a result
    W = wl.glorot(np.random.Generator(np.random.Philox(key=seed + 1)), d_in, d_out, (d_in, d_out))
    b = wl.random_matrix(1, d_out, seed + 2)[0] if bias else None
    Z = torch.full((n, ldz), 777.0, dtype=torch.float32, device="cuda")
    Hn.transform(Hn.dev(H), d_in, Hn.dev(W), Hn.dev(b) if bias else None, relu, out=Z)
    torch.cuda.synchronize()
    Zh = Z.cpu().numpy()
    assert np.all(Zh[:, d_out:] == 777.0)                  # padding columns untouched
    return H, W, b, Zh[:, :d_out]


@pytest.mark.parametrize("n,d_in,d_out,ldh,ldz,relu,bias", [
    (1000, 37, 5, 37, 5, False, True),          # everything unaligned, skinny output
    (333, 100, 256, 128, 256, False, True),     # GAT first round shape
    (700, 1204, 256, 1216, 512, True, True),    # SAGE large: K tail of 4
    (129, 2866, 64, 2880, 128, True, True),     # tiny-SAGE hidden layer
    (257, 512, 41, 512, 41, False, True),       # classifier, odd width
    (515, 256, 188, 256, 192, False, False),    # GAT last round, no bias
    (64, 16, 32, 16, 32, True, False),          # exactly one tile, one K step
    (1, 3, 300, 3, 300, False, True),           # single row, more than one column tile
    (2049, 128, 7, 128, 32, False, True),
    # aligned shapes (the software-pipelined kernel): one, two, three and many K steps, with and without a K tail
    (130, 16, 256, 16, 256, False, True),
    (1500, 32, 256, 32, 256, True, True),
    (1500, 48, 200, 64, 256, True, True),
    (4000, 20, 128, 32, 128, False, True),
    (300, 36, 4, 48, 16, False, False),
    (777, 260, 96, 272, 96, True, True),
    (5000, 52, 64, 64, 64, False, True),
    (3001, 200, 32, 208, 32, True, False),
    (1000, 64, 192, 64, 192, True, True),        # the 192-column tile, full and partly used
    (1000, 40, 132, 48, 144, False, True),
])
def test_transform_matches_oracle(n, d_in, d_out, ldh, ldz, relu, bias):
    H, W, b, Z = run(n, d_in, d_out, ldh, ldz, relu, bias, seed=n + d_in)
    want = oracle.transform(H, d_in, W, b, relu)
    assert_close(Z, want, what="transform %dx%d->%d" % (n, d_in, d_out))


def test_transform_with_no_input_columns_is_the_bias():
    # an empty product: every row is act(b), and neither H nor W is read (both may be NULL)
    n, d_out = 300, 40
    b = Hn.dev(wl.random_matrix(1, d_out, 3)[0])
    Z = torch.full((n, 48), 777.0, dtype=torch.float32, device="cuda")
    for flags, want in ((0, b), (B.F_RELU, torch.clamp(b, min=0))):
        B.check(B.retexo_transform(n, 0, d_out, 0, 0, 0, b.data_ptr(), flags, Z.data_ptr(), 48, Hn._stream_ptr()), "transform")
        torch.cuda.synchronize()
        assert torch.equal(Z[:, :d_out], want.expand(n, d_out)) and bool((Z[:, d_out:] == 777.0).all())


def test_transform_identity_weight_is_exact_and_relu_clamps():
    n, d = 300, 96
    H = wl.random_matrix(n, d, 5)
    Z = Hn.transform(Hn.dev(H), d, Hn.dev(np.eye(d, dtype=np.float32)), None, False)
    assert np.array_equal(Z.cpu().numpy()[:, :d], H)
    Z = Hn.transform(Hn.dev(H), d, Hn.dev(np.eye(d, dtype=np.float32)), None, True)
    assert np.array_equal(Z.cpu().numpy()[:, :d], np.maximum(H, 0))


def test_transform_small_integers_are_exact():
    # products and sums of small integers are exact in fp32 in any order: checks operand indexing
    n, d_in, d_out = 400, 70, 130
    H = wl.random_matrix(n, d_in, 6, kind="smallint")
    W = wl.random_matrix(d_in, d_out, 7, kind="smallint")
    b = wl.random_matrix(1, d_out, 8, kind="smallint")[0]
    Z = Hn.transform(Hn.dev(H), d_in, Hn.dev(W), Hn.dev(b), False)
    assert np.array_equal(Z.cpu().numpy()[:, :d_out].astype(np.float64), oracle.transform(H, d_in, W, b))


def test_transform_is_deterministic_and_rejects_alias():
    n, d_in, d_out = 777, 200, 256
    H = Hn.dev(wl.random_matrix(n, d_in, 9))
    W = Hn.dev(wl.random_matrix(d_in, d_out, 10))
    a = Hn.transform(H, d_in, W, None, True).clone()
    b = Hn.transform(H, d_in, W, None, True)
    assert torch.equal(a, b)
    assert B.retexo_transform(n, d_in, d_in, H.data_ptr(), d_in, W.data_ptr(), 0, 0, H.data_ptr(), d_in) == B.E_ALIAS


def test_transform_aligned_and_unaligned_operands_give_the_same_bits():
    # 16-byte aligned rows and rows moved by one float (H and W) take different loads, never a different
    # order of arithmetic — in either kernel family
    n, d_in, d_out = 1111, 212, 256
    H = wl.random_matrix(n, d_in, 21)
    W = wl.random_matrix(d_in, d_out, 22)
    b = Hn.dev(wl.random_matrix(1, d_out, 23)[0])
    Ha, Wa = Hn.dev(H), Hn.dev(W)
    Hu = torch.empty(n * d_in + 1, dtype=torch.float32, device="cuda")[1:].view(n, d_in)
    Wu = torch.empty(d_in * d_out + 1, dtype=torch.float32, device="cuda")[1:].view(d_in, d_out)
    Hu.copy_(Ha)
    Wu.copy_(Wa)
    assert Hu.data_ptr() % 16 != 0 and Wu.data_ptr() % 16 != 0
    za = Hn.transform(Ha, d_in, Wa, b, True)
    zu = Hn.transform(Hu, d_in, Wu, b, True)
    assert torch.equal(za, zu)
