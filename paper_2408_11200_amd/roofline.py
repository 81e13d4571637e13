"""Work and traffic models for the B-spline layer.

`paper_sol` restates the paper's speed-of-light model (section "Performance
Benchmarking": compute model, best/worst-case memory models) so that Table 2
can be re-derived; the `mi355x_*` helpers apply the same idea to the forward +
backward path of this library on one MI355X.
"""

# MI355X nominal figures (AMD public numbers): 256 CUs at 2.4 GHz.
MI355X_HBM_BYTES_PER_S = 8.0e12
MI355X_FP32_VECTOR_FLOPS = 157.3e12          # packed fp32: 256 CU * 4 SIMD * 16 lanes * 2 (packed) * 2 flop * 2.4 GHz
MI355X_FP32_VECTOR_FLOPS_UNPACKED = 78.6e12  # one v_fma_f32 per lane per clock: half of the above
MI355X_FP32_MATRIX_FLOPS = 157.3e12


def paper_sol(N, d_in, d_out, K, G, p_flop, p_bw, s=4):
    """Paper's model: F = N*d_in*d_out*c_k with c_k = 2K(K+1); best-case bytes stream every unique
    coefficient once, worst-case bytes fetch K coefficients per edge.  Returns times in seconds."""
    c_k = 2 * K * (K + 1)
    flops = N * d_in * d_out * c_k
    b_best = s * (N * (d_in + d_out) + d_in * d_out * (G + K))
    b_worst = s * (N * (d_in + d_out) + N * d_in * d_out * K)
    t_c = flops / p_flop
    t_mb = b_best / p_bw
    t_mw = b_worst / p_bw
    return {"t_compute": t_c, "t_mem_best": t_mb, "t_mem_worst": t_mw,
            "t_sol_best": max(t_c, t_mb), "t_sol_worst": max(t_c, t_mw)}


def edge_evals(B, n_in, n_out):
    return B * n_in * n_out


def algorithmic_flops_per_edge(K, base_on_valu=True):
    """Minimum vector work per (sample, input, output) triple for forward + backward:
    K FMAs each for the spline value, dL/dx and dL/dcoef (w_s folded into the coefficients),
    plus one FMA each for the base term in forward, dL/dx and dL/dw_b."""
    return 6 * K + (6 if base_on_valu else 0)


def algorithmic_hbm_bytes(B, n_in, n_out, G, k, s=4):
    """Best-case HBM traffic of forward + backward: x read twice, gy once, y and gx written;
    coefficients and the two scale matrices read twice and their gradients written once."""
    return s * (B * (3 * n_in + 2 * n_out) + 3 * n_in * n_out * (G + k + 2))
