"""dsv_check_block_tables: the opt-in validation of block-table entries (the entry points trust
them).  The expected result is recomputed on the host with numpy from the same table."""
import numpy as np
import pytest

from workloads import gen

pytestmark = pytest.mark.gpu


def _expected(tables, tokens, num_blocks):
    S, M = tables.shape
    need = np.where(tokens > 0, (tokens.astype(np.int64) + 15) // 16, 0)
    col = np.arange(M)[None, :]
    used = col < np.minimum(need, M)[:, None]
    bad = used & ((tables < 0) | (tables >= num_blocks))
    bad[:, 0] |= (tokens < 0) | (need > M)
    flat = np.flatnonzero(bad)
    return int(bad.sum()), int(flat[0]) if len(flat) else 0x7fffffff


def _run(tables, tokens, num_blocks):
    import torch
    import paper_2504_09285_amd as dsv
    res = torch.full((2,), -5, dtype=torch.int32, device="cuda")
    dsv.dsv_check_block_tables(torch.from_numpy(np.ascontiguousarray(tables, np.int32)).cuda(),
                               torch.from_numpy(np.ascontiguousarray(tokens, np.int32)).cuda(), num_blocks, res)
    torch.cuda.synchronize()
    return tuple(int(x) for x in res.cpu().numpy())


def test_a_generated_table_is_clean_and_planted_entries_are_found():
    b = gen.config2(shrink=4)
    nb = int(b.k_pool.shape[0])
    tables, tokens = b.block_tables.copy(), b.ctx_lens.copy()
    assert _run(tables, tokens, nb) == (0, 0x7fffffff) == _expected(tables, tokens, nb)
    # entries past a row's context are never read and may hold anything
    for i in range(tables.shape[0]):
        tables[i, (int(tokens[i]) + 15) // 16:] = -77
    assert _run(tables, tokens, nb) == (0, 0x7fffffff)
    # one entry equal to num_blocks, one negative, one huge: all inside their rows' contexts
    rng = np.random.default_rng(7)
    rows = rng.choice(tables.shape[0], 3, replace=False)
    for r, v in zip(rows, (nb, -1, 2 ** 31 - 1)):
        tables[r, int(rng.integers((int(tokens[r]) + 15) // 16))] = v
    got = _run(tables, tokens, nb)
    assert got == _expected(tables, tokens, nb) and got[0] == 3
    # a pool one block smaller makes every use of the last block an offence
    got = _run(b.block_tables, b.ctx_lens, nb - 1)
    assert got == _expected(b.block_tables, b.ctx_lens, nb - 1)


def test_rows_wider_than_the_table_and_edge_shapes():
    tables = np.arange(12, dtype=np.int32).reshape(3, 4)
    assert _run(tables, np.array([64, 1, 0]), 12) == (0, 0x7fffffff)
    assert _run(tables, np.array([65, 1, 0]), 12) == _expected(tables, np.array([65, 1, 0]), 12) == (1, 0)
    assert _run(tables, np.array([16, -3, 40]), 12) == _expected(tables, np.array([16, -3, 40]), 12) == (1, 4)
    assert _run(tables, np.array([64, 64, 64]), 5) == _expected(tables, np.array([64, 64, 64]), 5) == (7, 5)
    wide = np.zeros((2, 1000), np.int32)
    wide[1, 999] = 9
    assert _run(wide, np.array([16000, 16000]), 9) == (1, 1999)


def test_hand_off_tables_of_config_1():
    """The destination table of a hand-off is the receiver's choice (its placement): checked with
    the token counts the chunks touch."""
    _, h = gen.config1()
    tok = np.zeros(h.dst_tables.shape[0], np.int32)
    for seq, t0, n, _ in h.chunks:
        tok[seq] = max(tok[seq], t0 + n)
    nb = int(h.dst_k.shape[1])
    assert _run(h.dst_tables, tok, nb) == (0, 0x7fffffff)
    assert _run(h.dst_tables, tok, 1)[0] == _expected(h.dst_tables, tok, 1)[0] > 0
