"""Helpers shared by the GPU parity tests: upload a workload, call the C ABI, fetch results."""
import numpy as np
import torch

import paper_2509_08309_amd as H
from paper_2509_08309_amd import workloads as W

TOL = 4e-3          # max abs error of the fp16 output against the fp64 checker
SENTINEL = 0x7BFF   # fp16 65504: rows the library must not touch keep this bit pattern


class Dev:
    """A workload resident on the GPU plus the ABI shape that describes it."""

    def __init__(self, w: W.Workload):
        assert torch.cuda.is_available(), "GPU tests need a GPU"
        H.binding.load()
        self.w = w
        dev = torch.device("cuda:0")
        self.q = w.q.to(dev)
        self.k = w.k_cache.to(dev)
        self.v = w.v_cache.to(dev)
        self.bt = torch.from_numpy(w.block_table).to(dev)
        self.sl = torch.from_numpy(w.seq_lens).to(dev)
        s = w.spec
        self.shape = H.make_shape(s.batch, s.n_q_heads, s.n_kv_heads, s.head_dim,
                                  w.block_table.shape[1])
        self.scale = s.scale

    def heads(self, head_ids):
        hid = np.asarray(head_ids, dtype=np.int32)
        return torch.from_numpy(hid).cuda(), len(hid)

    def new_out(self):
        B, Hq, D = self.q.shape
        out = torch.empty((B, Hq, D), dtype=torch.float16, device="cuda:0")
        out.view(torch.int16).fill_(np.int16(SENTINEL))
        return out

    def validate(self, head_ids):
        hid, n = self.heads(head_ids)
        H.check(H.hetis_attn_validate(self.shape, self.bt, self.sl, hid, n, self.w.num_blocks),
                "validate")

    def decode(self, head_ids, out=None):
        self.validate(head_ids)
        hid, n = self.heads(head_ids)
        out = self.new_out() if out is None else out
        H.check(H.hetis_attn_decode(self.shape, self.q, self.k, self.v, self.bt, self.sl, hid, n,
                                    self.scale, out), "hetis_attn_decode")
        torch.cuda.synchronize()
        no_expired_wait()
        return out

    def workspace(self, n_sel):
        """A fresh caller-owned workspace for hetis_attn_decode_ws, control words zeroed."""
        rc, nbytes = H.hetis_attn_decode_workspace_bytes(self.shape, n_sel)
        H.check(rc, "decode_workspace_bytes")
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        ws.fill_(0xAB)                    # stale contents everywhere ...
        H.check(H.hetis_attn_workspace_init(ws, nbytes), "workspace_init")   # ... then the init call
        return ws

    def decode_ws(self, head_ids, ws, out=None, stream=None, sync=True, hid=None):
        """`hid`: the (tensor, count) of self.heads(head_ids), which a caller that does not
        synchronise must keep alive until the stream has passed the call."""
        hid, n = self.heads(head_ids) if hid is None else hid
        out = self.new_out() if out is None else out
        H.check(H.hetis_attn_decode_ws(self.shape, self.q, self.k, self.v, self.bt, self.sl, hid, n,
                                       self.scale, out, ws, ws.numel(), stream), "hetis_attn_decode_ws")
        if sync:
            torch.cuda.synchronize()
            no_expired_wait(ws)
        return out

    def split(self, head_ids, chunk_tokens, max_seq_len, fill=float("nan")):
        self.validate(head_ids)
        hid, n = self.heads(head_ids)
        s = self.w.spec
        C = H.hetis_attn_split_num_chunks(max_seq_len, chunk_tokens)
        assert C > 0
        rc, ob, lb = H.hetis_attn_split_workspace_bytes(self.shape, n, max_seq_len, chunk_tokens)
        H.check(rc, "workspace_bytes")
        r = s.group_size
        o_p = torch.full((s.batch, n, C, r, s.head_dim), fill, dtype=torch.float32, device="cuda:0")
        lse_p = torch.full((s.batch, n, C, r), fill, dtype=torch.float32, device="cuda:0")
        assert o_p.numel() * 4 == ob and lse_p.numel() * 4 == lb
        H.check(H.hetis_attn_decode_split(self.shape, self.q, self.k, self.v, self.bt, self.sl,
                                          hid, n, self.scale, chunk_tokens, max_seq_len, o_p,
                                          lse_p), "hetis_attn_decode_split")
        torch.cuda.synchronize()
        no_expired_wait()
        return o_p, lse_p

    def merge(self, o_p, lse_p, head_ids, chunk_tokens, max_seq_len, out=None):
        hid, n = self.heads(head_ids)
        out = self.new_out() if out is None else out
        H.check(H.hetis_attn_merge(self.shape, o_p, lse_p, self.sl, hid, n, chunk_tokens,
                                   max_seq_len, out), "hetis_attn_merge")
        torch.cuda.synchronize()
        return out


def no_expired_wait(ws=None):
    """The workspace's error word is zero: no bounded wait inside a kernel gave up (ws None: the
    library-owned workspace)."""
    rc, flags = H.hetis_attn_workspace_status(ws)
    assert rc == 0 and flags == 0, f"a wait inside a kernel expired: status {rc}, flags {flags:#x}"


def partials_as_rows(o_p: torch.Tensor, lse_p: torch.Tensor):
    """Library layout [B, S, C, r, D] / [B, S, C, r] -> row-major [B, S*r, C, D] / [B, S*r, C] (fp64)."""
    B, S, C, r, D = o_p.shape
    o = as_f64(o_p).transpose(0, 1, 3, 2, 4).reshape(B, S * r, C, D)
    lse = as_f64(lse_p).transpose(0, 1, 3, 2).reshape(B, S * r, C)
    return o, lse


def rows_as_partials(o_rows, lse_rows, r):
    """Inverse of partials_as_rows for numpy arrays; returns float32 arrays in library layout."""
    B, SR, C, D = o_rows.shape
    S = SR // r
    o = o_rows.reshape(B, S, r, C, D).transpose(0, 1, 3, 2, 4)
    lse = lse_rows.reshape(B, S, r, C).transpose(0, 1, 3, 2)
    return np.ascontiguousarray(o, dtype=np.float32), np.ascontiguousarray(lse, dtype=np.float32)


def bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def as_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().astype(np.float64)


def selected_rows(spec: W.WorkloadSpec, head_ids):
    r = spec.group_size
    return sorted(g * r + i for g in head_ids for i in range(r))


def unselected_rows(spec: W.WorkloadSpec, head_ids):
    sel = set(selected_rows(spec, head_ids))
    return [h for h in range(spec.n_q_heads) if h not in sel]


def check_rows(out: torch.Tensor, ref: np.ndarray, rows, tol=TOL, what="") -> float:
    """Every element of the listed head rows of every sequence against the checker's fp64
    result: none still holds the sentinel the output was filled with (a row the library never
    wrote would otherwise pass as a finite number), none is NaN, all within `tol`."""
    rows = list(rows)
    raw = bits(out)[:, rows]
    assert (raw != SENTINEL).all(), f"{what}: {int((raw == SENTINEL).all(axis=-1).sum())} selected rows never written"
    got = as_f64(out)[:, rows]
    assert not np.isnan(got).any(), f"{what}: NaN in a selected row"
    err = float(np.abs(got - ref[:, rows]).max()) if got.size else 0.0
    assert err <= tol, f"{what}: max abs err {err:.3e} > {tol}"
    return err


def check_mask(out: torch.Tensor, ref: np.ndarray, mask: np.ndarray, tol=TOL, what="") -> float:
    """As check_rows for a boolean [B, Hq] mask of rows (per-request head subsets); rows outside
    the mask must still hold the sentinel."""
    raw = bits(out)
    assert (raw[mask] != SENTINEL).all(), f"{what}: a named row was never written"
    assert (raw[~mask] == SENTINEL).all(), f"{what}: rows that no pair names were written"
    got = as_f64(out)[mask]
    assert not np.isnan(got).any(), f"{what}: NaN in a named row"
    err = float(np.abs(got - ref[mask]).max()) if got.size else 0.0
    assert err <= tol, f"{what}: max abs err {err:.3e} > {tol}"
    return err


def host_copy(w: W.Workload) -> W.Workload:
    """The same workload with its tensors in host memory (what the checker reads)."""
    return W.Workload(w.spec, w.seq_lens, w.block_table, w.num_blocks, w.q.cpu(), w.k_cache.cpu(),
                      w.v_cache.cpu(), w.head_ids)
