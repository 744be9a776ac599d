"""Algorithmic work of the expert layer: the FLOP and byte counts the benchmark divides by.

The paper's resource-allocation section counts, per batch element, C_f = 4*k*S*H*D_e FLOP
for an expert FFN made of two GEMMs (up and down projection) over the k*S routed tokens,
and 2*S*k*H bytes of bf16 per dispatch or combine, giving an FFN intensity of 2*D_e FLOP
per communicated byte.  With R routed rows (R = k*S when all experts are local) that is
2*R*d*f FLOP per GEMM.  The SwiGLU FFN built here has three weight matrices, so the
forward is 6*R*d*f and the backward (dgrad + wgrad of each) 12*R*d*f.
Padding rows, tail tiles and recomputation count as zero useful work.
"""


def gemm_flops(R, d, f, n_matrices=1):
    """FLOP of n_matrices [R,d]x[d,f]-shaped products."""
    return 2.0 * R * d * f * n_matrices


def paper_two_gemm_ffn_flops(k, S, H, De, b=1):
    """C_f of the resource-allocation section (two-matrix FFN, forward)."""
    return gemm_flops(b * k * S, H, De, 2)


def expert_fwd_flops(R, d, f):
    return gemm_flops(R, d, f, 3)


def expert_bwd_flops(R, d, f):
    return gemm_flops(R, d, f, 6)


def layer_flops(R, d, f):
    return expert_fwd_flops(R, d, f) + expert_bwd_flops(R, d, f)


def routed_bytes(R, d, elem_bytes=2):
    """Bytes of the routed rows themselves (the paper's 2*S*k*H for bf16 with R = k*S)."""
    return R * d * elem_bytes


def dispatch_bytes(U, R, T, k, d, elem_bytes):
    """Row mover, token order -> expert order: read each token that has a local slot once (U),
    write each routed row once (R), read inv (and nothing else)."""
    return (U + R) * d * elem_bytes + 4 * (R + T * k)


def combine_bytes(R, T, k, d, elem_bytes):
    """Row mover, expert order -> token order: read R rows, write T rows, read inv and gates."""
    return (R + T) * d * elem_bytes + 8 * T * k


def expert_composite_bound_s(rows_per_expert, d, f, elem_bytes, peak_flops, peak_bw):
    """Lower bound on the expert forward+backward time that accounts for experts too small to be
    compute bound: sum over experts of max(FLOP_e / peak_flops, bytes_e / peak_bw), where
    bytes_e counts the expert's weights (read by the forward and by the backward, gradients
    written once: 9*d*f elements) and the minimum activation traffic of its rows (6*d + 14*f
    elements per row over the six GEMMs)."""
    total = 0.0
    for rows in rows_per_expert:
        flops = 18.0 * rows * d * f
        byts = (9.0 * d * f + rows * (6.0 * d + 14.0 * f)) * elem_bytes
        total += max(flops / peak_flops, byts / peak_bw)
    return total
