"""The paper's closed-form cost relations (sections 3.1.1 and 3.1.3).

Test infrastructure only (see the package docstring).
"""


def kernel_time(t_launch, t_comp, t_mem, t_comm, t_non_overlap, t_sync):
    """Section 3.1.1: launch + the longest of the overlapped phases + what cannot overlap + sync."""
    return t_launch + max(t_comp, t_mem, t_comm) + t_non_overlap + t_sync


def tile_compute_time(m, n, K, R):
    """Section 3.1.3: an m x n output tile costs 2*m*n*K flops over the whole reduction, at R flop/s."""
    return 2.0 * m * n * K / R


def tile_comm_time(m, n, s, B):
    """Section 3.1.3: sending the m x n tile of s-byte elements over a B byte/s link."""
    return float(s) * m * n / B


def hiding_threshold_K(s, R, B):
    """Section 3.1.3: communication hides under compute once K >= s*R / (2*B)."""
    return s * R / (2.0 * B)


def comm_ratio(t_gemm, t_fused):
    """Table 3's last column: the share of the fused kernel's time not covered by the bare GEMM."""
    return (t_fused - t_gemm) / t_fused
