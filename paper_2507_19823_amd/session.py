"""Buffer plumbing for one layer's decode state: torch owns the memory, libhca does the work.

Nothing here computes anything; it allocates the tensors the C ABI expects and forwards calls.
"""
import math

import torch

from . import binding as B


class LayerState:
    """Key cache, scores, selection, accumulated scores and slot->value-row map of one layer."""

    def __init__(self, batch, n_q_heads, n_kv_heads, capacity, bits=4, group=32, k_max=1024, m_max=None,
                 device="cuda", want_z=False, workspace=None):
        self.shape = B.make_shape(batch, n_q_heads, n_kv_heads, capacity, bits, group)
        self.batch, self.hq, self.hkv, self.cap = batch, n_q_heads, n_kv_heads, capacity
        self.rows = batch * n_kv_heads
        self.k_max = k_max
        self.m_max = capacity if m_max is None else m_max
        nbytes = B.hca_kcache_bytes(self.shape)
        if nbytes == 0:
            raise B.HcaError("hca_kcache_bytes", -2)
        self.device = device
        self.kcache = torch.empty(nbytes, dtype=torch.uint8, device=device)
        self.sel = torch.empty(batch, n_kv_heads, capacity, dtype=torch.float32, device=device)
        self.z = torch.empty(batch, n_q_heads, capacity, dtype=torch.float32, device=device) if want_z else None
        self.idx_buf = torch.full((batch * n_kv_heads * k_max,), -1, dtype=torch.int32, device=device)
        self.k = k_max
        self.idx = self.idx_buf.view(batch, n_kv_heads, k_max)
        self.count = torch.zeros(batch, n_kv_heads, dtype=torch.int32, device=device)
        self.acc = torch.zeros(batch, n_kv_heads, capacity, dtype=torch.float32, device=device)
        self.pos = torch.arange(capacity, dtype=torch.int32, device=device).repeat(batch, n_kv_heads, 1).contiguous()
        self.y = torch.zeros(batch, n_q_heads, 128, dtype=torch.float32, device=device)
        if workspace is None:
            workspace = torch.empty(B.hca_workspace_bytes(self.shape, k_max, self.m_max), dtype=torch.uint8,
                                    device=device)
        self.ws = workspace
        self.n = [0] * batch
        self.sm_scale = 1.0 / math.sqrt(128.0)

    def quantize(self, k_new, value_row0=None, stream=None):
        """Append k_new [B,Hkv,T,D]; with value_row0 (one int per sequence) also resets acc and sets pos."""
        T = k_new.shape[2]
        if value_row0 is None:
            B.hca_quantize_keys(self.shape, self.kcache, k_new, T, self.n, None, None, None, stream)
        else:
            B.hca_quantize_keys(self.shape, self.kcache, k_new, T, self.n, self.acc, self.pos, value_row0, stream)
        self.n = [x + T for x in self.n]

    def score(self, q, stream=None):
        B.hca_score_qkeys(self.shape, self.kcache, q, self.n, self.sel, self.z, None, stream)

    def topk(self, k, stream=None):
        assert k <= self.k_max
        self.k = k
        self.idx = self.idx_buf[: self.rows * k].view(self.batch, self.hkv, k)   # row stride k
        B.hca_topk(self.shape, self.sel, self.n, k, self.idx, self.count, self.ws, stream)

    def score_topk(self, q, k, stream=None):
        """score + topk as one call that never writes the per-token scores (self.sel is left untouched)."""
        assert k <= self.k_max
        self.k = k
        self.idx = self.idx_buf[: self.rows * k].view(self.batch, self.hkv, k)
        B.hca_score_topk(self.shape, self.kcache, q, self.n, k, self.idx, self.count, self.ws, stream)

    def attend(self, q, v_host, n_host_rows, v_hbm, use_acc=True, gather_stream=None, stream=None):
        hs = 0 if v_host is None else v_host.shape[2]
        ds = 0 if v_hbm is None else v_hbm.shape[2]
        B.hca_sparse_attend(self.shape, self.kcache, q, self.idx, self.count, self.k, self.pos, v_host, hs,
                            n_host_rows, v_hbm, ds, self.sm_scale, self.y, self.acc if use_acc else None,
                            self.ws, gather_stream, stream)

    def evict(self, M, n_protect, kept=None, stream=None, spare=None):
        """In place, or (spare = (kcache, acc, pos) of the same shapes) out of place followed by a swap;
        the old buffers are returned as the next spare."""
        if spare is None:
            B.hca_evict(self.shape, self.kcache, self.acc, self.pos, self.n, M, n_protect, kept, self.ws,
                        None, None, None, stream)
            out = None
        else:
            B.hca_evict(self.shape, self.kcache, self.acc, self.pos, self.n, M, n_protect, kept, self.ws,
                        spare[0], spare[1], spare[2], stream)
            out = (self.kcache, self.acc, self.pos)
            self.kcache, self.acc, self.pos = spare
        self.n = [min(x, M) for x in self.n]
        return out

    def export(self):
        cb = 128 * self.shape.bits // 8
        ng = 128 // self.shape.group
        codes = torch.zeros(self.batch, self.hkv, self.cap, cb, dtype=torch.uint8, device=self.device)
        scale = torch.zeros(self.batch, self.hkv, self.cap, ng, dtype=torch.float16, device=self.device)
        zero = torch.zeros(self.batch, self.hkv, self.cap, ng, dtype=torch.float16, device=self.device)
        B.hca_export_kcache(self.shape, self.kcache, self.n, codes, scale, zero)
        return codes, scale, zero
