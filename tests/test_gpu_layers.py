"""GPU parity: ReLU, scaling and sign-activation layers through the C ABI against the oracle: output
labels (garbler's zero labels and evaluator's active labels) and every ciphertext byte."""
import numpy as np
import pytest
import torch

import workloads
from gpu_util import both, upload_bundle, assert_bundle_equal, assert_tables_equal
from oracle import plain

pytestmark = pytest.mark.gpu


def run_activation(k, kind, X, repeat=1, rule=0, layer=6, elem_base=0, first_wire=500, digits=None, exact=True, lam=None,
                   default_digits=False, in_place=False):
    from paper_2302_06361_amd import Labels, Layer, RELU, SCALE, SIGN
    if default_digits:      # the library picks the digit set; the oracle is built from what it reports
        from paper_2302_06361_amd import Context
        from oracle import capi
        from gpu_util import SEED
        ctx = Context(workloads.PRIMES[:k], SEED, None, rule)
        orc = capi.Oracle(workloads.PRIMES[:k], ctx.digits, SEED, rule)
    else:
        ctx, orc = both(k, rule, digits=digits, lam=lam)
    n = len(X)
    zero = [orc.input_labels(first_wire, n, i) for i in range(k)]
    act = [orc.encode(i, np.asarray(X), zero[i]) for i in range(k)]
    if kind == "relu":
        r0, rt = orc.relu_garble(layer, zero, elem_base)
        r = orc.relu_eval(layer, act, rt, elem_base)
        lay = Layer(RELU, layer, n, elem_base=elem_base)
        want = plain.relu(X, orc.P)
    elif kind == "scale":
        r0, rt = orc.scale_garble(layer, zero, repeat, elem_base)
        r = orc.scale_eval(layer, act, rt, repeat, elem_base)
        lay = Layer(SCALE, layer, n, elem_base=elem_base, repeat=repeat)
        want = plain.scale(X, orc.P, repeat)
    else:
        r0, rt = orc.signact_garble(layer, zero, elem_base)
        r = orc.signact_eval(layer, act, rt, elem_base)
        lay = Layer(SIGN, layer, n, elem_base=elem_base)
        want = plain.sign_act(X, orc.P)
    oe, tb, sb = ctx.layer_sizes(lay)
    assert oe == n and tb == rt.size
    tz, ta = upload_bundle(ctx, zero), upload_bundle(ctx, act)
    oz, oa = (tz, ta) if in_place else (Labels(ctx, n, zero=True), Labels(ctx, n, zero=True))      # in place: out over in
    tables = torch.zeros(max(tb, 4), dtype=torch.uint8, device=ctx.device)[:tb]
    scratch = torch.zeros(sb + 256, dtype=torch.uint8, device=ctx.device)
    ctx.garble_layer(lay, tz, oz, tables, scratch)
    scratch.fill_(0xA5)       # the evaluator must not depend on what the garbler left in scratch
    ctx.eval_layer(lay, ta, tables, oa, scratch)
    torch.cuda.synchronize()
    assert_bundle_equal(oz, r0, kind + " zero labels")
    assert_tables_equal(tables, rt, kind + " tables")
    assert_bundle_equal(oa, r, kind + " active labels")
    vals, valid = orc.decode(r, r0)
    assert valid.all() and (not exact or (vals == plain.to_signed(want, orc.P)).all())


@pytest.mark.parametrize("k", [2, 3, 4])
@pytest.mark.parametrize("kind", ["relu", "scale", "sign"])
def test_activation_every_value_small_bases(k, kind):
    P = int(np.prod(workloads.PRIMES[:k]))
    run_activation(k, kind, np.arange(P))


@pytest.mark.parametrize("kind,repeat", [("relu", 1), ("scale", 1), ("scale", 6), ("sign", 1)])
def test_activation_base8(kind, repeat):
    P = int(np.prod(workloads.PRIMES[:8]))
    g = np.random.default_rng(8)
    X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P // 2 + 1, P - 1], g.integers(0, P, 295)])   # 301: two blocks, ragged
    run_activation(8, kind, X, repeat=repeat, elem_base=123456789)


@pytest.mark.parametrize("kind,repeat", [("relu", 1), ("scale", 2)])
def test_activation_base12(kind, repeat):
    P = int(np.prod(workloads.PRIMES[:12]))
    g = np.random.default_rng(12)
    X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P - 1], g.integers(0, P, 95)])
    run_activation(12, kind, X, repeat=repeat, elem_base=2 ** 32 + 7)


def test_activation_one_gate_per_lane_digit_path(monkeypatch):
    """the digit gates of the sign gadget through the general gate kernels (one gate per lane) instead of the fused
    kernels: the path that gadgets below the size thresholds take; thresholds forced through their tuning hooks"""
    monkeypatch.setenv("DASH_FUSED_MIN_ELEMS_GARBLE", "1000000000")
    monkeypatch.setenv("DASH_FUSED_MIN_ELEMS_EVAL", "1000000000")
    P8 = int(np.prod(workloads.PRIMES[:8]))
    X = np.random.default_rng(77).integers(0, P8, 300)
    run_activation(8, "relu", X)
    run_activation(8, "scale", X, repeat=2)
    P7 = int(np.prod(workloads.PRIMES[:7]))
    run_activation(7, "scale", np.random.default_rng(78).integers(0, P7, 200), repeat=2, digits=workloads.DIGITS[7])


@pytest.mark.parametrize("k", [7, 8, 9, 12])
def test_activation_bank_replicated_tables_forced(monkeypatch, k):
    """the instantiations with bank-replicated AES tables (taken by launches of 2^20 lanes and more: the wide layers
    of configs 2 and 5 and of the model shapes f and F) forced for small layers, for the gate kernels and for the fused
    digit garbler alike: every byte of ReLU and scaling layers of the 7-, 8-, 9- and 12-prime bases (the four digit sets
    with compile-time kernels) against the oracle"""
    monkeypatch.setenv("DASH_BANKED_MIN_LANES", "1")
    monkeypatch.setenv("DASH_DIGITS_BANKED_MIN_LANES", "1")
    monkeypatch.setenv("DASH_WIDE_MAX_LANES", "0")       # the evaluator's digit gates fused per residue, as on wide layers
    monkeypatch.setenv("DASH_GARBLE_FEW_ROWS", "0")      # and the garbler's launches in the forms for many rows
    P = int(np.prod(workloads.PRIMES[:k]))
    g = np.random.default_rng(100 + k)
    X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P - 1], g.integers(0, P, 1296)])     # 1301 values: ragged tiles of 1024 lanes
    run_activation(k, "relu", X, elem_base=2 ** 31 + 3)
    run_activation(k, "scale", X[:333], repeat=2, elem_base=77)


@pytest.mark.parametrize("wide,sums", [("0", "1"), ("1000000000000", "1"), ("1000000000000", "0")])
def test_activation_both_forms_of_the_evaluators_digit_gates(monkeypatch, wide, sums):
    """The evaluator runs the digit gates of a sign gadget one lane per (element, residue, digit) for gadgets over few
    elements and one lane per (element, residue) with n hashes, fused with the scaling gadget's cast step, for the rest;
    the garbler likewise has a form of its launches for few rows (a lane per row of the digit gates; gates of different
    output moduli in one launch, each job with its modulus' compile-time code) and one for many: both forms forced on
    the same layers (4 KB tables), compile-time and run-time digit sets, every byte against the oracle.  With one digit
    gate per lane and a digit set with compile-time moduli the launch also forms the sums over the residues (the free
    gates of the mixed-radix addition) and stores no digit wire; that is switched off in the third case."""
    monkeypatch.setenv("DASH_WIDE_MAX_LANES", wide)
    monkeypatch.setenv("DASH_GARBLE_FEW_ROWS", wide)
    monkeypatch.setenv("DASH_QUAD_MAX_LANES", wide)      # carry chain: four lanes per element that share each AES, or one
    monkeypatch.setenv("DASH_SUM_IN_LAUNCH", sums)       # one digit gate per lane: the launch adds up the digit wires itself, or not
    for k in (7, 8, 9, 12):
        P = int(np.prod(workloads.PRIMES[:k]))
        X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P - 1], np.random.default_rng(300 + k).integers(0, P, 296)])
        run_activation(k, "relu", X, elem_base=5)
        run_activation(k, "scale", X, repeat=3, elem_base=2 ** 32 + 1)
    P5 = int(np.prod(workloads.PRIMES[:5]))
    run_activation(5, "scale", np.random.default_rng(9).integers(0, P5, 300), repeat=2)       # run-time digit set
    run_activation(5, "sign", np.random.default_rng(10).integers(0, P5, 300))


def test_activation_floor_rule():
    P = int(np.prod(workloads.PRIMES[:5]))
    g = np.random.default_rng(5)
    run_activation(5, "relu", g.integers(0, P, 130), rule=1)
    run_activation(5, "scale", g.integers(0, P, 130), repeat=2, rule=1)


def test_activation_explicit_label_lengths():
    """label lengths passed per prime to dash_ctx_create (shorter and longer than either rule gives)"""
    P = int(np.prod(workloads.PRIMES[:5]))
    X = np.random.default_rng(31).integers(0, P, 140)
    lam = (64, 90, 17, 46, 3)
    run_activation(5, "relu", X, lam=lam)
    run_activation(5, "scale", X, repeat=2, lam=lam)
    run_activation(5, "sign", X, lam=lam)


@pytest.mark.parametrize("k", [5, 7, 9, 10])
def test_activation_default_digit_sets(k):
    """no digit set given: the library searches one (prod(d) >= k P, smallest tables); the oracle, built from the
    digits the library reports, must agree on every byte, and the sign must be exact (decoded values checked)"""
    P = int(np.prod(workloads.PRIMES[:k]))
    g = np.random.default_rng(40 + k)
    X = np.concatenate([[0, 1, P // 2 - 1, P // 2, P // 2 + 1, P - 1], g.integers(0, P, 194)])
    run_activation(k, "relu", X, default_digits=True)
    run_activation(k, "scale", X, repeat=2, default_digits=True)


def test_activation_in_place():
    """output bundle = input bundle, for the garbler and for the evaluator: the garbler writes the output's zero labels
    only after its last read of the input's"""
    P = int(np.prod(workloads.PRIMES[:8]))
    X = np.random.default_rng(61).integers(0, P, 200)
    for kind, rep in (("relu", 1), ("scale", 3), ("sign", 1)):
        run_activation(8, kind, X, repeat=rep, in_place=True)


@pytest.mark.parametrize("n", [63, 64, 65, 129])
def test_activation_sizes_around_a_block_of_the_small_gadget_kernels(n):
    """the kernels for gadgets over few elements work on blocks of 64 elements (digit gates that add up their outputs) and
    on quads of lanes (carry chain, half gate): sizes just below, at and above a block"""
    P = int(np.prod(workloads.PRIMES[:8]))
    X = np.random.default_rng(500 + n).integers(0, P, n)
    run_activation(8, "relu", X, elem_base=7)
    run_activation(8, "scale", X, repeat=2, elem_base=2 ** 33)


def test_activation_single_element():
    run_activation(8, "relu", np.array([12345]))
    run_activation(8, "scale", np.array([9699689]), repeat=3)


def test_reduced_accuracy_digit_sets():
    """fewer mixed-radix digits (M < k P, Appendix, Approximated Garbled Sign): the approximated gadgets, bit for
    bit against the oracle, for the 3-digit set of the 8-prime base and a 2-digit set of a small base"""
    P8 = int(np.prod(workloads.PRIMES[:8]))
    g = np.random.default_rng(77)
    X = np.concatenate([g.integers(0, P8, 300), [0, 1, P8 // 2 - 1, P8 // 2, P8 - 1], P8 // 2 - 1 - g.integers(0, 20000, 100)])
    for kind, rep in (("relu", 1), ("scale", 2), ("sign", 1)):
        run_activation(8, kind, X, repeat=rep, digits=workloads.DIGITS_REDUCED[8], exact=False)
    P4 = int(np.prod(workloads.PRIMES[:4]))
    run_activation(4, "relu", np.arange(P4), digits=(4, 15), exact=False)


def test_empty_layer_calls_are_accepted():
    """zero elements: every layer kind returns without launching anything"""
    from paper_2302_06361_amd import Labels, Layer, RELU, SCALE, SIGN, DENSE, CONV2D, SUMPOOL
    ctx, orc = both(3)
    t = Labels(ctx, 0)
    w = ctx.weights_prepare(np.ones((4, 8), np.int32))
    for lay in (Layer(RELU, 1, 0), Layer(SCALE, 2, 0, repeat=2), Layer(SIGN, 3, 0),
                Layer(DENSE, 4, 0, in_c=8, out_c=4, weights=w),
                Layer(CONV2D, 5, 0, in_h=2, in_w=2, in_c=2, out_c=4, kh=1, kw=1, stride=1, pad=0, weights=w),
                Layer(SUMPOOL, 6, 0, in_h=2, in_w=2, in_c=2)):
        oe, tb, sb = ctx.layer_sizes(lay)
        assert tb == 0
        ctx.garble_layer(lay, t, t, None, None)
        ctx.eval_layer(lay, t, None, t, None)
    ctx.encode(torch.zeros(0, dtype=torch.int64, device=ctx.device), t, t)
    ctx.decode(t, t, torch.zeros(0, dtype=torch.int64, device=ctx.device), torch.zeros(0, dtype=torch.uint8, device=ctx.device))
    torch.cuda.synchronize()
