"""A third description of the block table, for the tests only: it never moves
a byte.  It remembers what the "model" wrote for every token of every request
and can check any implementation's images through that implementation's own
block mapping."""
import numpy as np

from tests import kvviews as V

NONE, DIRTY, FULL, SYNCED, HOST = 0, 1, 2, 3, 4


class LogicalKV:
    def __init__(self, shape, layout, seed=0):
        self.shape, self.layout = shape, layout
        self.rng = np.random.default_rng(seed)
        self.tokens = {}   # req -> uint16 array [n_tokens, L, 2, H, D]

    def token_dims(self):
        s = self.shape
        return (s.n_layers, 2, s.n_kv_heads, s.head_dim)

    def grow(self, req, n_tokens):
        """Draw the KV of n_tokens new tokens; returns them [n, L, 2, H, D]."""
        new = self.rng.integers(0, 1 << 16, size=(n_tokens,) + self.token_dims(), dtype=np.uint16)
        old = self.tokens.get(req)
        self.tokens[req] = new if old is None else np.concatenate([old, new])
        return new

    def drop(self, req):
        self.tokens.pop(req, None)

    def write_new_tokens(self, cache_u16, block_ids, old_len, new):
        """What the model does after an append: store the new tokens' KV in HBM."""
        cv = V.hbm_view(self.shape, cache_u16)
        P = self.shape.block_size
        for k in range(new.shape[0]):
            tok = old_len + k
            cv[:, :, block_ids[tok // P], tok % P] = new[k]

    def check(self, table_blocks, cache_u16, pool_u16, counts=None, reqs=None):
        """table_blocks(req) -> dict or None.  Every request's tokens must be
        readable through its mapping, and the mapping must be consistent."""
        s = self.shape
        P = s.block_size
        cv = V.hbm_view(s, cache_u16)
        pv = V.pool_view(s, pool_u16, self.layout)
        used_hbm, used_slots = set(), set()
        for req, toks in self.tokens.items():
            b = table_blocks(req)
            assert b is not None, f"request {req} vanished"
            n_tok = toks.shape[0]
            assert b["len"] == n_tok
            nb = (n_tok + P - 1) // P
            assert len(b["ids"]) == nb
            for i in range(nb):
                lo, hi = i * P, min(n_tok, (i + 1) * P)
                want = toks[lo:hi].transpose(1, 2, 0, 3, 4)      # [L,2,t,H,D]
                st, hid, sl = b["states"][i], b["ids"][i], b["slots"][i]
                full = (i + 1) * P <= n_tok
                if b["resident"]:
                    assert st in (DIRTY, FULL, SYNCED) and hid >= 0
                    assert np.array_equal(cv[:, :, hid, :hi - lo], want), (req, i, "HBM content")
                    if st == FULL:
                        assert full
                    if st == DIRTY:
                        assert not full
                    if st == SYNCED:   # the DRAM copy must be valid too
                        assert sl >= 0
                        assert np.array_equal(pv[:, :, sl, :hi - lo], want), (req, i, "DRAM copy of a synced block")
                else:
                    assert st == HOST and hid == -1 and sl >= 0
                    assert np.array_equal(pv[:, :, sl, :hi - lo], want), (req, i, "DRAM content")
                if hid >= 0:
                    assert hid not in used_hbm, "HBM block owned twice"
                    used_hbm.add(hid)
                if sl >= 0:
                    assert sl not in used_slots, "host slot owned twice"
                    used_slots.add(sl)
        if counts is not None:
            assert counts["free_hbm"] == s.n_hbm_blocks - len(used_hbm)
            assert counts["free_slots"] == s.n_host_slots - len(used_slots)
