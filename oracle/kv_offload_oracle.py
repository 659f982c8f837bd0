"""CPU oracle for moving one request's paged K/V out of and back into the pool.  TEST INFRASTRUCTURE.

Only tests may import this file; it shares no code with the package.

Algorithm 2 (memory-aware execution) offloads a waiting task's KV cache to host memory once it
has waited T_max, and the task resumes later from that copy.  What is moved is plain bytes, so
the definition is an index map.  The pool is [layer][page][head][slot][head_dim]; request b's
token t lives in page block_table[b][t // page_size], slot t % page_size.  The packed form of
a request with n cached tokens holds whole pages, ceil(n / page_size) of them:
    packed[layer][0 = K, 1 = V][j][head][slot][head_dim] = pool[layer][block_table[b][j]][head][slot][:]
Reloading writes the same values into the pages that a (possibly different) block table now
assigns to the request; slots past the n-th token carry whatever the source page held.
Memory check: a task that needs `need` more bytes may start when used + need <= threshold.
"""
import numpy as np


def n_pages_of(n_tokens, page_size):
    return (n_tokens + page_size - 1) // page_size


def pack(k_pool, v_pool, table_row, n_tokens):
    n_layers, _, n_heads, page, dh = k_pool.shape
    npg = n_pages_of(n_tokens, page)
    out = np.empty((n_layers, 2, npg, n_heads, page, dh), dtype=k_pool.dtype)
    for l in range(n_layers):
        for j in range(npg):
            out[l, 0, j] = k_pool[l, table_row[j]]
            out[l, 1, j] = v_pool[l, table_row[j]]
    return out


def unpack(packed, k_pool, v_pool, table_row):
    n_layers, _, npg = packed.shape[:3]
    for l in range(n_layers):
        for j in range(npg):
            k_pool[l, table_row[j]] = packed[l, 0, j]
            v_pool[l, table_row[j]] = packed[l, 1, j]


def memory_available(used, need, threshold):
    return used + need <= threshold
