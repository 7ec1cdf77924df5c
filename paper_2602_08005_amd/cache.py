"""Device pools of the compressed cache and host-side placement helpers.

Pure data placement: allocating the pools the C library describes, building
block / reference tables, and copying logical (token-major) arrays into or out
of the paged layout using the offset tables the library exports.  No arithmetic
of the method lives here.
"""
from __future__ import annotations

import numpy as np

from . import binding as B


class PagedCache:
    """Pools + per-sequence maps for `batch` sequences.

    page_ids[b] / ref_slots[b] give, per sequence, the pool page of each logical
    page and the pool slot of each reference ordinal (contiguous if omitted).
    """

    def __init__(self, dims: B.Dims, max_batch: int, max_new_tokens: int, max_seq_len: int,
                 device="cuda", page_ids=None, ref_slots=None):
        import torch
        self.torch = torch
        self.dims = dims
        self.layout = B.paged_layout(dims, max_batch, max_new_tokens, max_seq_len)
        self.device = device
        L = self.layout
        self.latent_pool = torch.zeros(L.latent_pool_bytes // 2, dtype=torch.int16, device=device)
        self.idx_pool = torch.zeros(L.idx_pool_bytes // 4, dtype=torch.int32, device=device)
        self.ref_pool = torch.zeros(L.ref_pool_bytes // 2, dtype=torch.int16, device=device)
        self.ref_inv_norm = torch.zeros(L.ref_norm_pool_bytes // 4, dtype=torch.float32, device=device)
        P, S = dims.page_tokens, dims.ref_stride
        self.max_pages = -(-max_seq_len // P)
        self.max_refs = -(-max_seq_len // S)
        bt = np.zeros((max_batch, self.max_pages), dtype=np.int32)
        rt = np.zeros((max_batch, self.max_refs), dtype=np.int32)
        for b in range(max_batch):
            if page_ids is None:
                bt[b] = np.arange(b * self.max_pages, (b + 1) * self.max_pages) % dims.n_pages
            else:
                bt[b, :len(page_ids[b])] = page_ids[b]
            if ref_slots is None:
                rt[b] = np.arange(b * self.max_refs, (b + 1) * self.max_refs) % dims.n_ref_slots
            else:
                rt[b, :len(ref_slots[b])] = ref_slots[b]
        self.block_tables_host, self.ref_tables_host = bt, rt
        self.block_tables = torch.from_numpy(bt).to(device)
        self.ref_tables = torch.from_numpy(rt).to(device)
        self.q4 = dims.latent_bits == 4
        self.off = [] if self.q4 else [B.latent_block_offsets(dims, s).astype(np.int64) for s in range(L.n_streams)]
        self.q4_off = [tuple(a.astype(np.int64) for a in B.q4_block_offsets(dims, s)) for s in range(L.n_streams)] \
            if self.q4 else []
        self.compress_ws = torch.empty(max(L.compress_ws_bytes, 256), dtype=torch.uint8, device=device)
        self.decode_ws = torch.empty(max(L.decode_ws_bytes, 256), dtype=torch.uint8, device=device)

    # -- logical <-> paged copies (host numpy in, device pools updated) ---------------------------
    def _latent_index(self, b: int, t0: int, t1: int, stream: int) -> np.ndarray:
        d, L = self.dims, self.layout
        t = np.arange(t0, t1)
        page = self.block_tables_host[b, t // d.page_tokens].astype(np.int64)
        base = page[:, None] * L.latent_page_stride + np.arange(d.n_kv_heads)[None, :] * L.latent_head_stride \
            + stream * L.latent_stream_stride                                  # [n, H]
        return base[:, :, None] + self.off[stream][t % d.page_tokens][:, None, :]   # [n, H, r]

    def _idx_index(self, b: int, t0: int, t1: int) -> np.ndarray:
        d, L = self.dims, self.layout
        t = np.arange(t0, t1)
        page = self.block_tables_host[b, t // d.page_tokens].astype(np.int64)
        ks = max(int(d.top_k), 1)
        ii = page[:, None, None] * L.idx_page_stride + np.arange(d.n_kv_heads)[None, :, None] * L.idx_head_stride \
            + np.arange(ks)[None, None, :] * L.idx_slot_stride + (t % d.page_tokens)[:, None, None]
        return ii if ks > 1 else ii[:, :, 0]                 # [n, H] or, with top_k > 1 ordinal slots, [n, H, top_k]

    def _ref_index(self, b: int, j0: int, j1: int, kv: int) -> np.ndarray:
        d, L = self.dims, self.layout
        slot = self.ref_tables_host[b, j0:j1].astype(np.int64)
        return (np.arange(d.n_kv_heads)[None, :, None] * L.ref_head_stride + kv * L.ref_kv_stride
                + slot[:, None, None] * L.ref_slot_stride + np.arange(d.head_dim)[None, None, :])

    def put_sequence(self, b: int, idx, zb_k, zb_v, ref_k_bits, ref_v_bits, ref_inv_norm=None, t0: int = 0,
                     chunk: int = 16384):
        """Copy token-major arrays of sequence b (tokens t0..t0+n-1; references 0..n_ref-1) into the pools."""
        torch = self.torch
        n = idx.shape[0]
        for c0 in range(0, n, chunk):
            c1 = min(n, c0 + chunk)
            for stream, zb in enumerate((zb_k, zb_v)[: self.layout.n_streams]):
                if zb is None:
                    continue
                ii = torch.from_numpy(self._latent_index(b, t0 + c0, t0 + c1, stream).ravel()).to(self.device)
                vv = torch.from_numpy(np.ascontiguousarray(zb[c0:c1]).view(np.int16).ravel()).to(self.device)
                self.latent_pool[ii] = vv
            ii = torch.from_numpy(self._idx_index(b, t0 + c0, t0 + c1).ravel()).to(self.device)
            self.idx_pool[ii] = torch.from_numpy(np.ascontiguousarray(idx[c0:c1], dtype=np.int32).ravel()).to(self.device)
        if ref_k_bits is not None:
            nr = ref_k_bits.shape[0]
            for c0 in range(0, nr, chunk):
                c1 = min(nr, c0 + chunk)
                for kv, bits in enumerate((ref_k_bits, ref_v_bits)):
                    ii = torch.from_numpy(self._ref_index(b, c0, c1, kv).ravel()).to(self.device)
                    self.ref_pool[ii] = torch.from_numpy(
                        np.ascontiguousarray(bits[c0:c1]).view(np.int16).ravel()).to(self.device)
            if ref_inv_norm is not None:
                slot = self.ref_tables_host[b, :nr].astype(np.int64)
                ii = (np.arange(self.dims.n_kv_heads)[None, :] * self.layout.ref_norm_head_stride + slot[:, None])
                self.ref_inv_norm[torch.from_numpy(ii.ravel()).to(self.device)] = \
                    torch.from_numpy(np.ascontiguousarray(ref_inv_norm, dtype=np.float32).ravel()).to(self.device)

    def get_sequence(self, b: int, t0: int, t1: int):
        """Token-major copies (numpy) of tokens t0..t1-1 of sequence b: idx, zb_k, zb_v."""
        torch = self.torch
        out = []
        ii = torch.from_numpy(self._idx_index(b, t0, t1).ravel()).to(self.device)
        idx = self.idx_pool[ii].cpu().numpy().reshape(self._idx_index(b, t0, t1).shape)
        for stream in range(self.layout.n_streams):
            ii = torch.from_numpy(self._latent_index(b, t0, t1, stream).ravel()).to(self.device)
            out.append(self.latent_pool[ii].cpu().numpy().view(np.uint16)
                       .reshape(t1 - t0, self.dims.n_kv_heads, self.dims.rank))
        if len(out) == 1:
            out.append(out[0])
        return idx, out[0], out[1]

    # -- 4-bit latents (format stated with the pool layout in the library header) -------------------
    def _q4_index(self, b: int, t0: int, t1: int, stream: int = 0):
        """2-byte element indices of the code half-words [n, H, r] (+ nibble shifts [r]) and of the scale and zero
        point [n, H] of tokens t0..t1-1 in latent stream `stream` (0: scores-operand order; 1: value-operand order)."""
        d, L = self.dims, self.layout
        t = np.arange(t0, t1)
        page = self.block_tables_host[b, t // d.page_tokens].astype(np.int64)
        base = page[:, None] * L.latent_page_stride + np.arange(d.n_kv_heads)[None, :] * L.latent_head_stride \
            + stream * L.latent_stream_stride
        code_off, shift_off, sc_off, zp_off = self.q4_off[stream]           # the library's statement of the record layout
        tok = t % d.page_tokens
        code_el = base[:, :, None] + code_off[tok][:, None, :]
        return code_el, shift_off[0], base + sc_off[tok][:, None], base + zp_off[tok][:, None]

    def get_sequence_q4(self, b: int, t0: int, t1: int, stream: int = 0):
        """Token-major copies of the 4-bit records of tokens t0..t1-1 in one latent stream: idx [n, H], codes uint8
        [n, H, r], bf16 bits of scale and zero point [n, H]."""
        torch = self.torch
        code_el, shift, sc_el, zp_el = self._q4_index(b, t0, t1, stream)
        ii = torch.from_numpy(self._idx_index(b, t0, t1).ravel()).to(self.device)
        idx = self.idx_pool[ii].cpu().numpy().reshape(t1 - t0, self.dims.n_kv_heads)
        take = lambda el: self.latent_pool[torch.from_numpy(el.ravel()).to(self.device)].cpu().numpy().view(np.uint16) \
            .reshape(el.shape)
        codes = ((take(code_el) >> shift[None, None, :].astype(np.uint16)) & 0xF).astype(np.uint8)
        return idx, codes, take(sc_el), take(zp_el)

    def put_sequence_q4(self, b: int, idx, codes, scale_bits, zero_bits, ref_k_bits, ref_v_bits, t0: int = 0,
                        codes_v=None, scale_bits_v=None, zero_bits_v=None):
        """Copy token-major 4-bit records (tokens t0..t0+n-1; t0 and n should cover whole pages except at the
        sequence's end: the half-words that hold the codes are rebuilt from the arrays given) and the references into
        the pools.  The *_v arrays are the value stream of the two-stream layout."""
        torch = self.torch
        n = idx.shape[0]
        streams = [(codes, scale_bits, zero_bits)] + ([(codes_v, scale_bits_v, zero_bits_v)] if codes_v is not None else [])
        for stream, (cd, sb, zb) in enumerate(streams):
            code_el, shift, sc_el, zp_el = self._q4_index(b, t0, t0 + n, stream)
            flat = code_el.ravel()
            vals = (cd.astype(np.uint16) << shift[None, None, :].astype(np.uint16)).ravel()
            uniq, inv = np.unique(flat, return_inverse=True)
            words = np.zeros(len(uniq), dtype=np.uint16)
            np.bitwise_or.at(words, inv, vals)
            self.latent_pool[torch.from_numpy(uniq).to(self.device)] = torch.from_numpy(words.view(np.int16)).to(self.device)
            for el, bits in ((sc_el, sb), (zp_el, zb)):
                self.latent_pool[torch.from_numpy(el.ravel()).to(self.device)] = \
                    torch.from_numpy(np.ascontiguousarray(bits, dtype=np.uint16).view(np.int16).ravel()).to(self.device)
        self.put_sequence(b, idx, None, None, ref_k_bits, ref_v_bits, t0=t0)

    def get_refs(self, b: int, n_ref: int):
        torch = self.torch
        res = []
        for kv in range(2):
            ii = torch.from_numpy(self._ref_index(b, 0, n_ref, kv).ravel()).to(self.device)
            res.append(self.ref_pool[ii].cpu().numpy().view(np.uint16)
                       .reshape(n_ref, self.dims.n_kv_heads, self.dims.head_dim))
        slot = self.ref_tables_host[b, :n_ref].astype(np.int64)
        ii = (np.arange(self.dims.n_kv_heads)[None, :] * self.layout.ref_norm_head_stride + slot[:, None])
        nrm = self.ref_inv_norm[torch.from_numpy(ii.ravel()).to(self.device)].cpu().numpy() \
            .reshape(n_ref, self.dims.n_kv_heads)
        return res[0], res[1], nrm

    def status(self) -> int:
        """Status word of the last decode call on this cache's workspace (synchronises the device).  Diagnostic:
        non-zero means some output rows were recomputed by the library's slow exact kernel."""
        self.torch.cuda.synchronize()
        return int(self.decode_ws[:4].view(self.torch.int32)[0].item())

    def _keep(self, stream, *tensors):
        """Per-call device tensors (lengths, selections) are temporaries of the caller's current stream; when the
        call runs on another stream the allocator must not hand their memory out again before that stream is done."""
        if stream is not None:
            for t in tensors:
                if t is not None and hasattr(t, "record_stream"):
                    t.record_stream(stream)

    # -- calls ------------------------------------------------------------------------------------
    def compress(self, w_down_k, w_down_v, k_new, v_new, cu_new_host, len_before_host, stream=None,
                 first_seq: int = 0):
        """Compress new tokens of sequences first_seq .. first_seq+len(len_before_host)-1."""
        torch = self.torch
        cu = torch.tensor(np.asarray(cu_new_host, dtype=np.int32), device=self.device)
        lb = torch.tensor(np.asarray(len_before_host, dtype=np.int32), device=self.device)
        n = len(len_before_host)
        self._keep(stream, cu, lb)
        return B.compress(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool,
                          self.ref_inv_norm, self.block_tables[first_seq:first_seq + n],
                          self.ref_tables[first_seq:first_seq + n], w_down_k, w_down_v, k_new,
                          v_new, cu, cu_new_host, lb, len_before_host, self.compress_ws, stream)

    def compress_mlp(self, kind, w1, wg, b1, w2, k_new, v_new, cu_new_host, len_before_host, stream=None,
                     first_seq: int = 0):
        """compress() with the non-linear compressor (JOINT caches with 16-bit latents)."""
        torch = self.torch
        cu = torch.tensor(np.asarray(cu_new_host, dtype=np.int32), device=self.device)
        lb = torch.tensor(np.asarray(len_before_host, dtype=np.int32), device=self.device)
        n = len(len_before_host)
        self._keep(stream, cu, lb)
        return B.compress_mlp(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool,
                              self.ref_inv_norm, self.block_tables[first_seq:first_seq + n],
                              self.ref_tables[first_seq:first_seq + n], kind, w1, wg, b1, w2, k_new,
                              v_new, cu, cu_new_host, lb, len_before_host, self.compress_ws, stream)

    def decode_attn(self, w_up_k, w_up_v, q, seq_lens_host, scale, out=None, lse=None, seq_lens=None,
                    stream=None):
        torch = self.torch
        if seq_lens is None:
            seq_lens = torch.tensor(np.asarray(seq_lens_host, dtype=np.int32), device=self.device)
        if out is None:
            out = torch.empty_like(q)
        self._keep(stream, seq_lens, out)
        B.decode_attn(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool,
                      self.block_tables, self.ref_tables, w_up_k, w_up_v, q, seq_lens, seq_lens_host, scale,
                      out, lse, self.decode_ws, stream)
        return out

    def decode_attn_rope(self, w_up_k, w_up_v, q_rot, seq_lens_host, scale, rope_base, out=None, lse=None, stream=None):
        torch = self.torch
        seq_lens = torch.tensor(np.asarray(seq_lens_host, dtype=np.int32), device=self.device)
        if out is None:
            out = torch.empty_like(q_rot)
        self._keep(stream, seq_lens, out)
        B.decode_attn_rope(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool, self.block_tables,
                           self.ref_tables, w_up_k, w_up_v, q_rot, seq_lens, seq_lens_host, scale, rope_base, out, lse,
                           self.decode_ws, stream)
        return out

    def selection(self, positions_per_seq):
        """Page lists + token masks (device int32 tensors) for per-sequence arrays of selected token positions."""
        torch = self.torch
        P = self.dims.page_tokens
        lists = []
        for pos in positions_per_seq:
            pos = np.unique(np.asarray(pos, dtype=np.int64))
            pages, inv = np.unique(pos // P, return_inverse=True)
            masks = np.zeros(len(pages), dtype=np.int64)
            np.bitwise_or.at(masks, inv, 1 << (pos % P))
            lists.append((pages.astype(np.int32), masks.astype(np.int32)))
        stride = max(1, max(len(p) for p, _ in lists))
        sp = np.zeros((len(lists), stride), dtype=np.int32)
        sm = np.zeros((len(lists), stride), dtype=np.int32)
        n = np.zeros(len(lists), dtype=np.int32)
        for b, (p, m) in enumerate(lists):
            sp[b, :len(p)], sm[b, :len(p)], n[b] = p, m, len(p)
        return torch.from_numpy(sp).to(self.device), torch.from_numpy(sm).to(self.device), \
            torch.from_numpy(n).to(self.device), n

    def decode_attn_subset(self, w_up_k, w_up_v, q, seq_lens_host, positions_per_seq, scale, out=None, lse=None,
                           stream=None):
        torch = self.torch
        seq_lens = torch.tensor(np.asarray(seq_lens_host, dtype=np.int32), device=self.device)
        sp, sm, n_dev, n_host = self.selection(positions_per_seq)
        if out is None:
            out = torch.empty_like(q)
        self._keep(stream, seq_lens, sp, sm, n_dev, out)
        B.decode_attn_subset(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool,
                             self.block_tables, self.ref_tables, w_up_k, w_up_v, q, seq_lens, seq_lens_host,
                             sp, sm, n_dev, n_host, scale, out, lse, self.decode_ws, stream)
        return out

    def decode_attn_raw(self, w_up_k, w_up_v, q, seq_lens_host, raw_k, raw_v, raw_lens_host, scale,
                        positions_per_seq=None, out=None, lse=None, stream=None):
        """Attention over the cache (or the selected positions) plus raw_lens_host[b] raw tokens per sequence;
        raw_k / raw_v: device bf16 bits [batch, raw_cap, n_kv_heads, head_dim]."""
        torch = self.torch
        seq_lens = torch.tensor(np.asarray(seq_lens_host, dtype=np.int32), device=self.device)
        raw_lens = torch.tensor(np.asarray(raw_lens_host, dtype=np.int32), device=self.device)
        sel = self.selection(positions_per_seq) if positions_per_seq is not None else None
        if out is None:
            out = torch.empty_like(q)
        self._keep(stream, seq_lens, raw_lens, out, *(sel[:3] if sel is not None else ()))
        B.decode_attn_raw(self.dims, self.layout, self.latent_pool, self.idx_pool, self.ref_pool, self.block_tables,
                          self.ref_tables, w_up_k, w_up_v, q, seq_lens, seq_lens_host, raw_k, raw_v, raw_lens, scale,
                          out, lse, self.decode_ws, selection=sel, stream=stream)
        return out
