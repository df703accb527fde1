"""The quantization-error study (Section 4.3 "Effectiveness of Tensor Quantization"; RTN baseline of
Section 4.1) from the oracle alone: prints the table the design notes quote and pins its directions."""
from oracle import error_study


def test_study_table_and_directions(capsys):
    rows = error_study.table()
    with capsys.disabled():
        print()
        for r in rows:
            print("error study: %s %d-bit G%d levels=%d  reconstruction DecoQuant %.3f RTN %.3f | attention DecoQuant %.3f RTN %.3f" % r)
    by = {(r[1], r[3]): r for r in rows}
    for levels in (0, 1):
        _, _, _, _, rd, rr, ad, ar = by[4, levels]
        # the paper's claim, in direction: at 4 bits quantizing only the large tensor beats quantizing the matrix
        assert rd < 0.75 * rr and ad < ar
        assert rd < 0.2 and rr < 0.3
    # the level set that uses every code lowers the reconstruction error of both strategies
    for bits in (2, 4):
        assert by[bits, 1][4] < by[bits, 0][4] and by[bits, 1][5] < by[bits, 0][5]
    # at 2 bits the synthetic rows do not reproduce the paper's direction: reported, and pinned as
    # measured so that a change in the oracle that moves it is noticed
    assert by[2, 0][4] > by[2, 0][5]


def test_length_of_local_tensors_table(capsys):
    """Section 4.3 "Analysis of Length of Local Tensors" on the stand-ins: two, three and four local
    tensors.  The paper reports a lower error for n = 3 and 4 on real activations; on these rows the
    reconstruction error does not move (within 3 %), with independent tokens and with neighbouring
    tokens made alike: the per-row steps of the large tensor already absorb what a token-side tensor
    concentrates.  Reported as measured and pinned so that a change in the oracle that moves it shows."""
    rows = error_study.length_table()
    with capsys.disabled():
        print()
        for name, bits, group, rho, r in rows:
            print("length study: %s %d-bit G%d %s  reconstruction n=2 %.3f n=3 %.3f n=4 %.3f RTN %.3f | attention n=2 %.3f n=3 %.3f n=4 %.3f RTN %.3f"
                  % (name, bits, group, "as drawn" if rho == 0.0 else "AR(1) %.2f" % rho, r["n=2"][0], r["n=3"][0], r["n=4"][0],
                     r["rtn"][0], r["n=2"][1], r["n=3"][1], r["n=4"][1], r["rtn"][1]))
    for name, bits, group, rho, r in rows:
        for n in ("n=3", "n=4"):
            assert abs(r[n][0] - r["n=2"][0]) <= 0.03 * r["n=2"][0], (name, rho, n)
        if bits == 4:   # every tensor count beats quantizing the matrix itself, in both measures
            for n in ("n=2", "n=3", "n=4"):
                assert r[n][0] < 0.75 * r["rtn"][0] and r[n][1] < r["rtn"][1], (name, rho, n)
