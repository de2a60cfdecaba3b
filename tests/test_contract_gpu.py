"""GPU parity tests of fg_contract against the CPU oracle (nested mode loops in FP64)."""
import numpy as np
import pytest
import torch

from paper_2009_12263_amd import binding as fg
from paper_2009_12263_amd import workloads as W
from tests.parity import delenv, run_contract_case, setenv

pytestmark = pytest.mark.gpu
a, b, c, d, e, f = 0, 1, 2, 3, 4, 5


def say(msg):
    print("[case] " + msg, flush=True)


def test_config5a_256():
    """BASELINE config 5: C[a,b,c] = sum_d A[a,d,c] B[d,b], a=b=c=d=256, dense, first mode fastest."""
    ext = {a: 256, b: 256, c: 256, d: 256}
    say("5a ints, every entry"); run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True)
    say("5a floats, sampled"); run_contract_case(ext, [a, d, c], [d, b], [a, b, c], samples=8192)


def test_config5b_64():
    """C[a,b,c,d] = sum_{e,f} A[a,e,b,f] B[d,f,c,e], all extents 64."""
    ext = {a: 64, b: 64, c: 64, d: 64, e: 64, f: 64}
    say("5b ints sampled"); run_contract_case(ext, [a, e, b, f], [d, f, c, e], [a, b, c, d], ints=True, samples=8192)
    say("5b floats sampled"); run_contract_case(ext, [a, e, b, f], [d, f, c, e], [a, b, c, d], samples=8192)


def test_paper_contraction_full_size():
    """The contraction the paper times in Section 5.5: D_abc = sum_d A_bda B_dc with
    (a, b, c, d) = (64, 32, 2048, 2048), sampled."""
    ext = {a: 64, b: 32, c: 2048, d: 2048}
    say("paper contraction ints sampled"); run_contract_case(ext, [b, d, a], [d, c], [a, b, c], ints=True, samples=8192)
    say("paper contraction floats sampled"); run_contract_case(ext, [b, d, a], [d, c], [a, b, c], samples=8192)
    dummy = torch.zeros(64, dtype=torch.float16, device="cuda"); out = torch.zeros(64, dtype=torch.float32, device="cuda")
    plan = fg.fg_contract_plan([b, d, a], W.col_major_strides((32, 2048, 64)), dummy, [d, c], W.col_major_strides((2048, 2048)), dummy,
                               [a, b, c], W.col_major_strides((64, 32, 2048)), None, out, ext)
    assert plan == "gett_nn_128x128x64_deep", plan


def test_result_contiguous_along_the_second_row_mode():
    """A is contiguous along one row mode and the result along another (the shape of the paper's
    own example): the rows of a block tile are then fed to the matrix unit in a permuted order so
    that a store covers consecutive elements of the result.  Every entry, integer data (exact):
    leading extents 8, 16, 32 and 64 (the last too long for the permutation), row extents that
    no tile divides, three row modes, alpha/beta with the result updated in place."""
    say("leading 16, 6 of the next"); run_contract_case({a: 6, b: 16, c: 40, d: 64}, [b, d, a], [d, c], [a, b, c], ints=True)
    say("leading 8, 20 of the next"); run_contract_case({a: 20, b: 8, c: 72, d: 128}, [b, d, a], [d, c], [a, b, c], ints=True, beta=1.0)
    say("leading 32, 5 of the next, in place"); run_contract_case({a: 5, b: 32, c: 136, d: 64}, [b, d, a], [d, c], [a, b, c], ints=True, alpha=2.0, beta=-1.0, inplace=True)
    say("leading 32, 40 of the next, many tiles"); run_contract_case({a: 40, b: 32, c: 264, d: 192}, [b, d, a], [d, c], [a, b, c], ints=True)
    say("leading 64"); run_contract_case({a: 12, b: 64, c: 48, d: 64}, [b, d, a], [d, c], [a, b, c], ints=True)
    say("three row modes, result order a, e, b"); run_contract_case({a: 12, b: 16, c: 40, d: 64, e: 3}, [b, d, e, a], [d, c], [a, e, b, c], ints=True)
    say("B also a tensor, floats"); run_contract_case({a: 24, b: 16, c: 8, d: 64, e: 5, f: 2}, [b, d, a, f], [d, f, c, e], [a, b, c, e], alpha=0.5, beta=-2.0)


def test_every_tile_shape_in_the_contraction_kernels(monkeypatch):
    """The five block tiles of the contraction kernels (the last one the 128x128 tile with a ring of
    four buffers) forced in turn on contractions with a contiguous result (streaming stores), a
    permuted one, batch modes and a C operand: integer data, every entry exact.  The deep ring also
    over summed extents shorter than the ring and in all four layout pairs."""
    for tile in range(5):
        setenv(monkeypatch, "FG_FORCE_TILE", str(tile))
        say("tile %d" % tile)
        run_contract_case({a: 64, b: 72, c: 5, d: 192}, [a, d, c], [d, b], [a, b, c], ints=True)
        run_contract_case({a: 12, b: 16, c: 40, d: 320}, [b, d, a], [d, c], [a, b, c], ints=True, beta=1.0)
        run_contract_case({a: 40, b: 24, c: 3, d: 128, e: 2}, [a, d, c, e], [d, e, b], [a, e, b, c], ints=True, alpha=2.0, beta=-1.0)
    setenv(monkeypatch, "FG_FORCE_TILE", "4")
    for K in (8, 64, 136, 256, 520):
        say("deep ring, summed extent %d" % K)
        run_contract_case({a: 136, b: 24, c: 7, d: K}, [a, d, c], [d, b], [a, b, c], ints=True)
    say("deep ring, A and B contiguous along the summed mode / along the rows and columns")
    run_contract_case({a: 40, b: 136, c: 3, d: 320}, [d, a, c], [d, b], [a, b, c], ints=True, beta=1.0)
    run_contract_case({a: 40, b: 136, c: 3, d: 320}, [d, a, c], [b, d], [a, b, c], ints=True)
    run_contract_case({a: 40, b: 136, c: 3, d: 320}, [a, d, c], [b, d], [a, b, c], ints=True)
    delenv(monkeypatch, "FG_FORCE_TILE")


def test_ragged_extents_every_entry():
    """Row and column extents that no block tile divides: edge tiles of the strided kernels are
    predicated in the loads (zeros) and in the stores (dropped)."""
    say("5a-shaped ragged"); run_contract_case({a: 24, b: 5, c: 7, d: 64}, [a, d, c], [d, b], [a, b, c], ints=True)
    say("5a-shaped ragged floats beta"); run_contract_case({a: 40, b: 100, c: 9, d: 128}, [a, d, c], [d, b], [a, b, c], alpha=0.5, beta=-2.0)
    say("5b-shaped ragged"); run_contract_case({a: 16, b: 3, c: 5, d: 8, e: 64, f: 3}, [a, e, b, f], [d, f, c, e], [a, b, c, d], ints=True)
    say("paper-shaped ragged"); run_contract_case({a: 5, b: 8, c: 33, d: 64}, [b, d, a], [d, c], [a, b, c], ints=True)
    say("K-contiguous operands, odd rows and columns"); run_contract_case({a: 37, b: 3, c: 51, d: 128}, [d, a, b], [d, c], [a, b, c], ints=True)
    say("several tiles with a ragged tail"); run_contract_case({a: 72, b: 9, c: 301, d: 64}, [a, d, b], [d, c], [a, b, c], ints=True)
    say("result's fastest mode in B, ragged"); run_contract_case({a: 56, b: 136, d: 64}, [a, d], [b, d], [b, a], ints=True, beta=1.0)


def test_summed_extents_that_are_not_multiples_of_64():
    """The leading summed mode is walked in steps of 64; other extents leave a zero-filled
    remainder in the last step of each pass."""
    say("K-contiguous A and B, leading summed extent 40, second summed mode")
    run_contract_case({a: 37, c: 51, d: 40, e: 3}, [d, a, e], [d, e, c], [a, c], ints=True)
    say("M-contiguous A (5a-shaped), summed extent 104")
    run_contract_case({a: 72, b: 40, c: 3, d: 104}, [a, d, c], [d, b], [a, b, c], ints=True)
    say("summed extent 8")
    run_contract_case({a: 64, b: 64, d: 8}, [a, d], [d, b], [a, b], ints=True)
    say("5b-shaped with extents 72 and 5, floats")
    run_contract_case({a: 16, b: 4, c: 8, d: 8, e: 72, f: 5}, [a, e, b, f], [d, f, c, e], [a, b, c, d], alpha=0.5, beta=-2.0)
    say("both operands M/N-contiguous, odd summed extent 13")
    run_contract_case({a: 64, b: 72, d: 13, e: 3}, [a, d, e], [b, e, d], [a, b], ints=True)
    say("every summed mode has extent 1")
    run_contract_case({a: 64, b: 72, d: 1}, [a, d], [b, d], [a, b], ints=True)
    say("summed extent 200 with a batch mode, sampled floats")
    run_contract_case({a: 256, b: 200, d: 200, f: 6}, [a, d, f], [d, b, f], [a, b, f], samples=4000)


def test_batch_modes():
    """Modes present in A, B and C: an independent contraction per batch index (one launch)."""
    g, h = 6, 7
    say("batched matrix product C[m,n,g] = A[m,k,g] B[k,n,g]")
    run_contract_case({a: 72, b: 40, d: 64, g: 5}, [a, d, g], [d, b, g], [a, b, g], ints=True)
    say("batch mode first in B, last in A, middle in C, floats, beta")
    run_contract_case({a: 64, b: 24, c: 3, d: 128, g: 4}, [a, d, c, g], [d, g, b], [a, g, b, c], alpha=0.5, beta=-1.0)
    say("two batch modes, two summed modes")
    run_contract_case({a: 16, b: 8, e: 64, f: 2, g: 3, h: 2}, [a, e, g, f, h], [b, f, h, e, g], [a, b, g, h], ints=True)
    say("K-contiguous operands with a batch mode")
    run_contract_case({a: 37, c: 51, d: 128, g: 3}, [d, a, g], [d, c, g], [a, c, g], ints=True)
    say("64 batches of 256x256x256, sampled")
    run_contract_case({a: 256, b: 256, d: 256, g: 64}, [a, d, g], [d, b, g], [a, b, g], samples=8192)


def test_small_contractions_every_entry():
    say("5a-shaped small"); run_contract_case({a: 64, b: 64, c: 3, d: 64}, [a, d, c], [d, b], [a, b, c], ints=True)
    say("5b-shaped small"); run_contract_case({a: 16, b: 4, c: 8, d: 8, e: 64, f: 2}, [a, e, b, f], [d, f, c, e], [a, b, c, d], ints=True)
    say("5b-shaped small floats, alpha/beta"); run_contract_case({a: 16, b: 8, c: 8, d: 16, e: 64, f: 3}, [a, e, b, f], [d, f, c, e], [a, b, c, d], alpha=0.5, beta=-2.0)
    say("paper's D_abc = A_bda B_dc"); run_contract_case({a: 4, b: 32, c: 64, d: 128}, [b, d, a], [d, c], [a, b, c], ints=True)
    say("paper's contraction, floats, in place"); run_contract_case({a: 4, b: 32, c: 64, d: 128}, [b, d, a], [d, c], [a, b, c], beta=1.0, inplace=True)
    say("both operands contiguous along the summed mode"); run_contract_case({a: 64, b: 2, c: 64, d: 128}, [d, a, b], [d, c], [a, b, c], ints=True)
    say("result's fastest mode belongs to B"); run_contract_case({a: 64, b: 128, d: 64}, [a, d], [b, d], [b, a], ints=True)


def test_padded_strides():
    # A[a,d,c] with padded strides, B[d,b] padded, C[a,b,c] padded: untouched gaps are checked
    ext = {a: 64, b: 64, c: 2, d: 64}
    run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, stridesA=[1, 72, 72 * 64 + 8], stridesB=[1, 80], stridesC=[1, 68, 68 * 64 + 4])


def test_poisoned_gaps_of_strided_tensors():
    """The gaps that padded strides leave in A, B and Cin hold NaN: the result must not see them
    (integer-exact), also with ragged extents whose edge tiles read past the extents."""
    ext = {a: 64, b: 64, c: 2, d: 64}
    run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, stridesA=[1, 72, 72 * 64 + 8], stridesB=[1, 80], stridesC=[1, 68, 68 * 64 + 4], poison=True)
    run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, beta=2.0, stridesA=[1, 72, 72 * 64 + 8], stridesB=[1, 80], stridesC=[1, 68, 68 * 64 + 4], poison=True)
    ext = {a: 40, b: 24, c: 3, d: 72}
    run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, beta=-1.0, stridesA=[1, 48, 48 * 72 + 16], stridesB=[1, 80], stridesC=[1, 44, 44 * 24 + 8], poison=True)
    # A contiguous along the summed mode
    run_contract_case(ext, [d, a, c], [d, b], [a, b, c], ints=True, stridesA=[1, 80, 80 * 40 + 8], stridesB=[1, 88], stridesC=[1, 44, 44 * 24 + 8], poison=True)


def test_descriptions_only_the_general_kernel_takes():
    """Contractions that miss a requirement of the tiled kernels: strides that are not multiples of
    8 elements, no contiguous mode at all, A and B contiguous along different summed modes, odd
    extents everywhere, an outer product, and a tensor of 2 GiB.  Integer-exact, every entry
    (sampled for the large one); gaps between strided elements hold NaN."""
    ext = {a: 64, b: 64, c: 2, d: 64}
    general = lambda *args: "general" in fg.fg_contract_plan(*args)
    t16, t32 = torch.empty(64, dtype=torch.float16, device="cuda"), torch.empty(64, dtype=torch.float32, device="cuda")
    sA, sB, sC = [1, 65, 65 * 64 + 3], [1, 67], [1, 65, 65 * 64 + 1]
    assert general([a, d, c], sA, t16, [d, b], sB, t16, [a, b, c], sC, None, t32, ext)
    say("general: odd strides"); run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, beta=2.0, stridesA=sA, stridesB=sB, stridesC=sC, poison=True)
    say("general: no unit stride"); run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, stridesA=[2, 130, 130 * 64], stridesB=[3, 200], stridesC=[2, 130, 130 * 64], poison=True)
    ext5 = {a: 40, b: 24, d: 16, e: 8}
    assert general([d, e, a], [1, 16, 128], t16, [e, d, b], [1, 8, 128], t16, [a, b], [1, 40], None, t32, ext5)
    say("general: different contiguous summed modes"); run_contract_case(ext5, [d, e, a], [e, d, b], [a, b], ints=True)
    say("general: odd extents, batch mode"); run_contract_case({a: 13, b: 7, c: 3, d: 29, e: 5}, [d, a, c, e], [b, d, e, c], [b, a, c], ints=True, beta=-1.0)
    say("general: outer product"); run_contract_case({a: 70, b: 33}, [a], [b], [a, b], ints=True)
    say("general: floats"); run_contract_case({a: 100, b: 50, d: 333}, [d, a], [b, d], [b, a], alpha=0.5, beta=1.5)
    say("general: A of 2 GiB, sampled")
    big = {a: 1 << 15, b: 24, d: 1 << 15}
    run_contract_case(big, [a, d], [d, b], [a, b], ints=True, samples=2000)


def test_delta_gives_mode_permutation():
    n = 64
    ext = {a: n, b: n, c: n, d: n}
    delta = torch.eye(n, dtype=torch.float16).reshape(-1)
    # C[a,b,c] = sum_d A[a,d,c] delta[d,b] = A[a,b,c]: checked against the oracle, which was pinned to this identity
    run_contract_case(ext, [a, d, c], [d, b], [a, b, c], ints=True, B_override=delta)


def test_seeded_random_contraction_sweep():
    """Sixty seeded random contractions: one or two row, column and summed modes, sometimes a
    batch mode, random order of the modes inside each tensor, random extents, nothing adjusted to
    the tiled kernels' requirements: descriptions they cannot take (no 8-aligned contiguous mode,
    A and B contiguous along different summed modes) run on the general kernel, and both kinds
    must occur.  Integer-valued, every entry compared."""
    import random
    rng = random.Random(5)
    kinds = {"tiled": 0, "general": 0}
    for case in range(60):
        labels = iter(range(100))
        rows = [next(labels) for _ in range(rng.randint(1, 2))]
        cols = [next(labels) for _ in range(rng.randint(1, 2))]
        sums = [next(labels) for _ in range(rng.randint(1, 2))]
        batch = [next(labels)] if rng.random() < 0.3 else []
        ext = {}
        for m in rows + cols:
            ext[m] = rng.choice([1, 2, 3, 5, 8, 12, 24, 40])
        for m in sums:
            ext[m] = rng.choice([1, 2, 3, 8, 16, 40, 72])
        for m in batch:
            ext[m] = rng.choice([2, 3])
        mA = rows + sums + batch
        mB = cols + sums + batch
        mC = rows + cols + batch
        rng.shuffle(mA); rng.shuffle(mB); rng.shuffle(mC)
        if case % 2 == 0:
            # make the description one the tiled kernels take: a non-batch first mode with an extent % 8 == 0
            for modes in (mA, mB):
                free = [m for m in modes if m not in batch]
                first = rng.choice(free)
                modes.remove(first); modes.insert(0, first)
            for first in (mA[0], mB[0]):
                if ext[first] % 8:
                    ext[first] = rng.choice([8, 16, 24, 40])
            if mA[0] in sums and mB[0] in sums and mA[0] != mB[0]:
                mB.remove(mA[0]); mB.insert(0, mA[0])
        dense = lambda ms: list(W.col_major_strides(tuple(ext[m] for m in ms)))
        fake = lambda dt: torch.empty(64, dtype=dt, device="cuda")      # only the alignment of the pointers matters
        plan = fg.fg_contract_plan(mA, dense(mA), fake(torch.float16), mB, dense(mB), fake(torch.float16), mC, dense(mC), None, fake(torch.float32), ext)
        kinds["general" if "general" in plan else "tiled"] += 1
        beta = rng.choice([0.0, 1.0, -0.5])
        say("sweep %d: A%s B%s C%s ext=%s beta=%g plan=%s" % (case, mA, mB, mC, ext, beta, plan))
        run_contract_case(ext, mA, mB, mC, alpha=rng.choice([1.0, 2.0, -1.0]), beta=beta, ints=True, seed=2000 + case)
    assert kinds["tiled"] >= 15 and kinds["general"] >= 15, kinds
