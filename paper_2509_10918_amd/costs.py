"""Algorithmic work of one ToMA layer call: closed-form flop and byte counts.

Used only to turn measured times into rates.  The flop formulas are the matrix-product counts of
the paper's complexity model (App. C: C_sub = N^2 d, C_proj = C_merge = C_unmerge = N D d per
sample, counted there in multiplications; here 2 flops per multiply-add) restricted to regions as
Sec. 4.3.1 describes, and the attention block of its FLOP table (App. G: Q/K/V projections plus
QK^T and PV).
"""


def attention_block_flops(B, L, C):
    """Q, K, V projections and the two attention products on L tokens of width C (App. G)."""
    return 2 * B * (3 * C * C * L + 2 * C * L * L)


def toma_overhead_flops(B, N, C, n_loc, d_loc):
    """Selection similarity + merge weights + merge + unmerge, all inside regions of n_loc tokens
    with d_loc destinations each (the 'Overhead' column of the paper's FLOP table)."""
    return 2 * B * N * C * (n_loc + 3 * d_loc)


def stage_flops(B, N, C, P, d_loc, merge_regions, T_extra=0):
    """Per-stage flops of one layer call (what the method must compute, not a dense layer)."""
    n_loc, D, R = N // P, P * d_loc, merge_regions
    L = D + T_extra
    per_gemm = 2 * B * N * D * C // R
    return {
        "similarity": 2 * B * N * n_loc * C,
        "weights": per_gemm,
        "merge": per_gemm,
        "qkv": 6 * B * L * C * C,
        "attention": 4 * B * L * L * C,
        "unmerge": per_gemm,
    }


def greedy_stream_bytes(B, P, n_loc, d_loc, elem=4):
    """Bytes Alg. 2 scans when every round after the first re-reads the region's similarity
    matrix: B*P regions, d_loc - 1 rounds, n_loc^2 entries each."""
    return B * P * (d_loc - 1) * n_loc * n_loc * elem
