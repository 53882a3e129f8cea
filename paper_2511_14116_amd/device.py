"""Device-side plumbing for one rank's share: torch owns the memory and the stream, the
library does every step of the path.  Used by the GPU tests, the smoke check and bench.py."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B

_KV_CODE = {"bf16": B.FS_KV_BF16, "fp8": B.FS_KV_FP8_E4M3}


class DeviceShare:
    """Q, the paged K/V pool (repacked into kernel order) and the page table on the GPU."""

    def __init__(self, shape: B.FsShape, q_bits: np.ndarray, kv: dict, sm_scale: float,
                 interleave_kv: bool = True, device: str = "cuda:0", v_range: int = B.FS_V_ANY,
                 scales_by_page: bool = True):
        if not torch.cuda.is_available():
            raise RuntimeError("DeviceShare needs a GPU; there is no CPU fallback")
        self.shape = shape
        self.device = torch.device(device)
        self.group = shape.n_q_heads // shape.n_kv_heads
        self.kv_dtype = _KV_CODE[kv["kv_dtype"]]
        self.q = torch.from_numpy(q_bits.view(np.int16)).to(self.device)
        tdt = torch.int16 if self.kv_dtype == B.FS_KV_BF16 else torch.uint8
        view = (lambda a: a.view(np.int16)) if self.kv_dtype == B.FS_KV_BF16 else (lambda a: a)
        n_slots, T, D = kv["k_pool"].shape
        slot_bytes = T * D * (2 if self.kv_dtype == B.FS_KV_BF16 else 1)
        stream = torch.cuda.current_stream().cuda_stream
        if interleave_kv:
            # K and V of a slot side by side: one 2*slot_bytes run per (page, head)
            self._pool = torch.empty((n_slots, 2, T * D), dtype=tdt, device=self.device)
            k_ptr, v_ptr = self._pool.data_ptr(), self._pool.data_ptr() + slot_bytes
            k_stride = v_stride = 2 * slot_bytes
        else:
            self._pool = (torch.empty((n_slots, T * D), dtype=tdt, device=self.device),
                          torch.empty((n_slots, T * D), dtype=tdt, device=self.device))
            k_ptr, v_ptr = self._pool[0].data_ptr(), self._pool[1].data_ptr()
            k_stride = v_stride = slot_bytes
        # the generator's pools are token-major; the library puts every slot into the order its kernels read
        for host, dst, is_v in ((kv["k_pool"], k_ptr, False), (kv["v_pool"], v_ptr, True)):
            src = torch.from_numpy(view(host)).to(self.device)
            B.fs_pack_kv_slots(src, slot_bytes, dst, k_stride, n_slots, self.kv_dtype, is_v, stream)
            torch.cuda.current_stream().synchronize()
            del src
        self.page_indptr = torch.from_numpy(kv["page_indptr"]).to(self.device)
        self.page_ids = torch.from_numpy(kv["page_ids"]).to(self.device)
        self.k_scale = self.v_scale = self.page_scales = None
        if kv["k_scale"] is not None:
            self.k_scale = torch.from_numpy(kv["k_scale"]).to(self.device)
            self.v_scale = torch.from_numpy(kv["v_scale"]).to(self.device)
            if scales_by_page:
                # the same scales in page-table order, (K, V) per page: what an engine keeps next to its page ids
                idx = self.page_ids.long()
                self.page_scales = torch.stack([self.k_scale[idx], self.v_scale[idx]], dim=1).contiguous()
        self.view = B.FsKvView(
            q=self.q.data_ptr(), k_pool=k_ptr, v_pool=v_ptr, k_slot_stride=k_stride, v_slot_stride=v_stride,
            k_scale=None if self.k_scale is None else self.k_scale.data_ptr(),
            v_scale=None if self.v_scale is None else self.v_scale.data_ptr(),
            page_indptr=self.page_indptr.data_ptr(), page_ids=self.page_ids.data_ptr(),
            kv_dtype=self.kv_dtype, sm_scale=float(sm_scale),
            page_scales=None if self.page_scales is None else self.page_scales.data_ptr(), v_range=int(v_range))
        self.kv_bytes = int(kv["page_indptr"][-1]) * 2 * slot_bytes
        self.n_items = self.n_pairs = 0

    def set_worklist(self, items: np.ndarray, pairs: np.ndarray, sched: np.ndarray, chunk_indptr: np.ndarray):
        """Upload a work list and size the partial and final output buffers for it."""
        self.n_items, self.n_pairs = len(items), len(pairs)
        G, D = self.group, self.shape.head_dim
        dev = self.device
        self.items = torch.from_numpy(np.ascontiguousarray(items).view(np.int32).reshape(-1, 8)).to(dev)
        self.sched = torch.from_numpy(np.ascontiguousarray(sched)).to(dev)
        self.chunk_indptr = torch.from_numpy(np.ascontiguousarray(chunk_indptr)).to(dev)
        self.part_o = torch.full((self.n_items * G, D), float("nan"), dtype=torch.float32, device=dev)
        self.part_lse = torch.full((self.n_items * G,), float("nan"), dtype=torch.float32, device=dev)
        self.out = torch.full((self.n_pairs * G, D), float("nan"), dtype=torch.float32, device=dev)
        self.lse = torch.full((self.n_pairs * G,), float("nan"), dtype=torch.float32, device=dev)

    def set_worklist_units(self, items: np.ndarray, pairs: np.ndarray, unit_indptr: np.ndarray, chunk_indptr: np.ndarray):
        """Upload a list cut into equal runs (fs_build_worklist_units) and size the outputs for it."""
        self.set_worklist(items, pairs, np.zeros(0, dtype=np.int32), chunk_indptr)
        self.n_units = len(unit_indptr) - 1
        self.unit_indptr = torch.from_numpy(np.ascontiguousarray(unit_indptr)).to(self.device)

    def run_units(self):
        B.fs_decode_attention_units(self.shape, self.view, self.items, self.n_items, self.unit_indptr, self.n_units,
                                    self.chunk_indptr, self.n_pairs, self.part_o, self.part_lse, self.out, self.lse,
                                    torch.cuda.current_stream().cuda_stream)

    def set_records(self, records: np.ndarray):
        """Upload launch records of the list that set_worklist / set_worklist_units brought."""
        assert len(records) == self.n_items
        self.records = torch.from_numpy(np.ascontiguousarray(records).view(np.int32).reshape(-1, 16)).to(self.device)

    def run_records(self, units: bool = False, merge_in_sweep: bool = False, claim: bool = False):
        """Sweep and merge in one call from launch records (one workgroup per record, or per unit; with ``claim``
        resident workgroups that claim the records in order).  With ``merge_in_sweep`` the pair counters are
        handed over and split pairs are merged by the sweep itself."""
        if merge_in_sweep and (not hasattr(self, "pair_counters") or len(self.pair_counters) < self.n_pairs):
            self.pair_counters = torch.zeros(max(self.n_pairs, 1), dtype=torch.int32, device=self.device)   # every call leaves them zero
        if claim and not hasattr(self, "claim"):
            self.claim = torch.zeros(2, dtype=torch.int32, device=self.device)   # every launch leaves them at zero
        B.fs_decode_attention_records(self.shape, self.view, self.records, self.n_items,
                                      self.unit_indptr if units else None, self.n_units if units else 0,
                                      self.chunk_indptr, self.n_pairs, self.part_o, self.part_lse, self.out, self.lse,
                                      self.pair_counters if merge_in_sweep else None, self.claim if claim else None,
                                      torch.cuda.current_stream().cuda_stream)

    def decode(self, use_sched: bool = True):
        B.fs_decode_attention(self.shape, self.view, self.items, self.sched if use_sched else None,
                              self.n_items, self.part_o, self.part_lse, torch.cuda.current_stream().cuda_stream)

    def decode_persistent(self, use_sched: bool = True):
        """The same partials by the persistent form of the sweep."""
        if not hasattr(self, "claim"):
            self.claim = torch.zeros(2, dtype=torch.int32, device=self.device)   # every launch leaves them at zero
        B.fs_decode_attention_persistent(self.shape, self.view, self.items, self.sched if use_sched else None,
                                         self.n_items, self.claim, self.part_o, self.part_lse,
                                         torch.cuda.current_stream().cuda_stream)

    def merge(self):
        B.fs_merge_lse(self.part_o, self.part_lse, self.chunk_indptr, self.n_pairs, self.group,
                       self.shape.head_dim, self.out, self.lse, torch.cuda.current_stream().cuda_stream)

    def run_fused(self, use_sched: bool = True, persistent: bool = True):
        """Sweep and merge in one library call; unsplit pairs get their final rows from the sweep.  With
        ``persistent`` the counters are handed over and the library takes the persistent sweep for long lists."""
        if persistent and not hasattr(self, "claim"):
            self.claim = torch.zeros(2, dtype=torch.int32, device=self.device)
        B.fs_decode_attention_fused(self.shape, self.view, self.items, self.sched if use_sched else None, self.n_items,
                                    self.chunk_indptr, self.n_pairs, self.part_o, self.part_lse,
                                    self.claim if persistent else None, self.out, self.lse,
                                    torch.cuda.current_stream().cuda_stream)

    def run(self, use_sched: bool = True, persistent: bool = False):
        if persistent:
            self.decode_persistent(use_sched)
        else:
            self.decode(use_sched)
        self.merge()

    # ---- chunked prefill: same Q / pool / page-table plumbing, another list and output shape ----
    def set_prefill_worklist(self, items: np.ndarray, sched: np.ndarray, chunk_indptr: np.ndarray, tile_tokens: int,
                             out_indptr: np.ndarray | None = None):
        """Upload a prefill item list and size the partial and final outputs for it.  ``out_indptr`` (first final
        row of every pair) is what the one-call form needs on top."""
        if out_indptr is not None:
            self.prefill_out_indptr = torch.from_numpy(np.ascontiguousarray(out_indptr)).to(self.device)
        dev = self.device
        self.n_prefill_items = len(items)
        self.n_prefill_tiles = len(chunk_indptr) - 1
        self.prefill_tile_tokens = int(tile_tokens)
        T = self.prefill_tile_rows = int(tile_tokens) * self.group
        D = self.shape.head_dim
        self.prefill_items = torch.from_numpy(np.ascontiguousarray(items).view(np.int32).reshape(-1, 8)).to(dev)
        self.prefill_sched = torch.from_numpy(np.ascontiguousarray(sched)).to(dev)
        self.prefill_chunk_indptr = torch.from_numpy(np.ascontiguousarray(chunk_indptr)).to(dev)
        self.prefill_part_o = torch.full((self.n_prefill_items * T, D), float("nan"), dtype=torch.float32, device=dev)
        self.prefill_part_lse = torch.full((self.n_prefill_items * T,), float("nan"), dtype=torch.float32, device=dev)
        self.prefill_out = torch.full((self.n_prefill_tiles * T, D), float("nan"), dtype=torch.float32, device=dev)
        self.prefill_lse = torch.full((self.n_prefill_tiles * T,), float("nan"), dtype=torch.float32, device=dev)

    def prefill_fused(self, use_sched: bool = True):
        """Attention and merge in one call; tiles of one chunk get their final rows from the kernel."""
        B.fs_prefill_attention_fused(self.shape, self.view, self.prefill_items, self.prefill_sched if use_sched else None,
                                     self.n_prefill_items, self.prefill_tile_tokens, self.prefill_chunk_indptr,
                                     self.n_prefill_tiles, self.prefill_out_indptr, self.prefill_part_o,
                                     self.prefill_part_lse, self.prefill_out, self.prefill_lse,
                                     torch.cuda.current_stream().cuda_stream)

    def prefill(self, use_sched: bool = True):
        """Per-item partials, then the split-K merge (the same fs_merge_lse the decode path uses)."""
        s = torch.cuda.current_stream().cuda_stream
        B.fs_prefill_attention(self.shape, self.view, self.prefill_items, self.prefill_sched if use_sched else None,
                               self.n_prefill_items, self.prefill_tile_tokens, self.prefill_part_o,
                               self.prefill_part_lse, s)
        B.fs_merge_lse(self.prefill_part_o, self.prefill_part_lse, self.prefill_chunk_indptr, self.n_prefill_tiles,
                       self.prefill_tile_rows, self.shape.head_dim, self.prefill_out, self.prefill_lse, s)
