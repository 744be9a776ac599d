"""The benchmark's FLOP/byte counters against the paper's analytic model
(resource-allocation section: C_f = b*4*k*S*H*D_e, volume b*2*S*k*H bytes, I_ffn = 2*D_e)."""
from paper_2605_11005_amd import counters as C


def test_paper_flop_and_byte_model():
    # the three evaluated models of the paper's model-configuration table at S = 4096
    for H, k, De in ((2048, 4, 1408), (2880, 4, 2880), (4096, 8, 1536)):
        S = 4096
        cf = C.paper_two_gemm_ffn_flops(k, S, H, De)
        assert cf == 4 * k * S * H * De
        vol = C.routed_bytes(k * S, H, 2)
        assert vol == 2 * S * k * H
        assert cf / vol == 2 * De                      # I_ffn
        R = k * S
        assert C.expert_fwd_flops(R, H, De) == 1.5 * cf  # third SwiGLU matrix
        assert C.layer_flops(R, H, De) == 18 * R * H * De


def test_row_mover_bytes():
    T, k, d, R, U = 1000, 8, 64, 900, 600
    assert C.dispatch_bytes(U, R, T, k, d, 2) == (U + R) * d * 2 + 4 * (R + T * k)
    assert C.combine_bytes(R, T, k, d, 2) == (R + T) * d * 2 + 8 * T * k
    assert C.dispatch_bytes(U, R, T, k, d, 2) <= 2 * R * d * 2 + 4 * (R + T * k)   # never above "rows moved"


def test_composite_bound_limits():
    d, f, P, BW = 7168, 2048, 2.5e15, 8e12
    # a large expert is compute bound, a tiny one is bound by its weights, an empty one still
    # has its gradient written (zeros) and nothing else is charged beyond the weights term
    big = C.expert_composite_bound_s([10000], d, f, 2, P, BW)
    assert abs(big - 18.0 * 10000 * d * f / P) < 1e-12
    tiny = C.expert_composite_bound_s([2], d, f, 2, P, BW)
    assert tiny > 100 * 18.0 * 2 * d * f / P and abs(tiny - (9 * d * f + 2 * (6 * d + 14 * f)) * 2 / BW) < 1e-12
    assert C.expert_composite_bound_s([10000, 2], d, f, 2, P, BW) == big + tiny
