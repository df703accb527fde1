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
