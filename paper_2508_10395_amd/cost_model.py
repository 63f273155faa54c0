"""Operation and byte counts of rematerialisation: the system-level model of Sec. 3.4 (arxiv 2508.10395).

Host arithmetic only, used by the benchmark to turn a measured time into a roofline fraction.  A
multiply-accumulate counts as two FLOPs, as in the paper.  Symbols follow the section: l cached tokens,
d hidden size, e bits per cached element, g query heads per KV head, P the ridge point (peak FLOP/s over
memory bytes/s) of the machine.
"""


def remat_flops(l, d, g=1):
    """FLOPs to rematerialise K and V of l cached tokens in one layer: 2*2*l*d^2 for MHA; with the latent
    cache of a grouped-query model the contraction is (d/g) x (d/g): 2*2*l*(d/g)^2."""
    r = d / g
    return 2.0 * 2.0 * l * r * r


def x_cache_bytes(l, d, e, g=1):
    """Bytes of cached X read per layer, codes only: e/8*l*d for MHA; for the latent cache the section's second
    equation uses e/8*l*d/g (its running text says twice that; the printed 40.6K follows the equation)."""
    return e / 8.0 * l * (d / g)


def kv_cache_bytes(l, d, e, g=1):
    """Bytes a KV cache of the same bit width reads per layer: 2*e/8*l*d/g."""
    return 2.0 * e / 8.0 * l * (d / g)


def max_remat_tokens(P, d, e, weight_bytes, g=1):
    """Largest l for which rematerialisation overlapped with loading `weight_bytes` of layer weights stays
    memory-bound: the solution of  P = remat_flops(l) / (x_cache_bytes(l) + weight_bytes)."""
    r = d / g
    return P * weight_bytes / (4.0 * r * r - P * e / 8.0 * r)


def layer_weight_bytes_llama2_7b(d):
    """fp16 weights of one Llama-2-7B layer as the section counts them: 2*12*d^2 bytes."""
    return 2.0 * 12.0 * d * d


def layer_weight_bytes_llama31_8b(d, g):
    """One Llama-3.1-8B layer incl. the SVD-decomposed Wk, Wv: 2*13*d^2 + 2*2*(d/g)^2 bytes."""
    return 2.0 * 13.0 * d * d + 2.0 * 2.0 * (d / g) ** 2


def cl_extra_flops(l, d):
    """XQuant-CL: adding the cached delta to the accumulator, 2*l*d per layer."""
    return 2.0 * l * d


def cl_gqa_flops(l, d, g):
    """XQuant-CL on a grouped-query model: up-projection by U_kv^T plus the K and V projections of the
    accumulator, 2*4*l*(d/g)*d per layer."""
    return 2.0 * 4.0 * l * (d / g) * d


# ---- the same counts for a launch of this library's kernels (batch B, so M = B*l token rows) -----------------

def remat_attn_flops(M, d, n_q_heads, n_kv_heads, head_dim):
    """xq_remat_attn_decode: the contraction X^ [Wk | Wv] of M rows (2*M*d*N, N = 2*n_kv_heads*head_dim; equals
    remat_flops summed over the batch when n_kv_heads*head_dim = d) plus scores and weighted sums (4*M*Hq*hd)."""
    N = 2 * n_kv_heads * head_dim
    return 2.0 * M * d * N + 4.0 * M * n_q_heads * head_dim


def remat_attn_algorithmic_bytes(M, d, bits, group, n_kv_heads, head_dim):
    """HBM bytes xq_remat_attn_decode has to move: packed codes, 2 x 16-bit metadata per group, one pass over
    the bf16 weights."""
    return M * d * bits / 8.0 + M * (d / group) * 4.0 + 2.0 * d * (2 * n_kv_heads * head_dim)


def quantize_bytes_per_element(bits, group, reads_accumulator=False):
    """xq_quantize_append (xq_cl_delta_quantize when the accumulator is read too): bf16 in, codes and metadata out."""
    return (4.0 if reads_accumulator else 2.0) + bits / 8.0 + 4.0 / group


def cl_accumulate_bytes_per_element(bits, group):
    """xq_cl_accumulate: bf16 accumulator read and written, codes and metadata read."""
    return 4.0 + bits / 8.0 + 4.0 / group
