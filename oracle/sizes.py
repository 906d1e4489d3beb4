"""Closed-form parameter and KV-cache counts (TEST INFRASTRUCTURE ONLY).

Table "Comparison of the memory footprint of MHA, MQA, GQA, MLA and Tucker
Attention": number of attention weights per layer and cached numbers per layer
for a sequence of N tokens.  Counts are in elements; multiply by bytes per
element and by the number of layers for the MB figures the result tables print.
The Tucker row is written for separate ranks (r1, r2, r3) and reduces to the
table's 2(nH r1 + 2 r d + r1 r^2) when r2 = r3 = r.
"""
from __future__ import annotations


def mha_params(d):
    return 4 * d * d


def mha_cache(N, d):
    return 2 * N * d


def gqa_params(d, d_head, n_groups):
    return 2 * d * d + 2 * n_groups * d_head * d


def gqa_cache(N, d_head, n_groups):
    return 2 * N * n_groups * d_head


def mla_params_train(d, dc, shared_kv):
    return d * d + (5 if shared_kv else 6) * d * dc


def mla_cache(N, dc, shared_kv):
    return (1 if shared_kv else 2) * N * dc


def tucker_params(d, n_heads, r1, r2, r3, shared_kv=False):
    """Pre- plus post-softmax tensors with tied ranks: cores, head factors, and the
    query/output factor (d x r2) and key/value factor (d x r3) of each tensor.
    With a shared key-value down-projection one d x r3 factor is dropped."""
    one = n_heads * r1 + (r2 + r3) * d + r1 * r2 * r3
    return 2 * one - (r3 * d if shared_kv else 0)


def tucker_cache(N, r3, shared_kv=False):
    return (1 if shared_kv else 2) * N * r3
