"""A synthetic workload copied to the GPU with the library's descriptor ready: the harness the GPU tests, the
smoke run and the benchmark share.  It only allocates tensors and forwards to the binding."""
import torch

from . import hcsa


class DeviceWorkload:
    """A synth.Workload copied to the GPU, with the library's descriptor ready."""

    def __init__(self, w, device="cuda:0"):
        self.w = w
        self.device = torch.device(device)
        self.q, self.k, self.v = (t.to(self.device) for t in (w.q, w.k, w.v))
        self.cu_q = torch.from_numpy(w.cu_q).to(self.device)
        self.cu_kv = torch.from_numpy(w.cu_kv).to(self.device)
        self.cu_k = torch.from_numpy(w.cu_k).to(self.device)
        self.seq_mode = torch.from_numpy(w.seq_mode).to(self.device)
        self.max_q = int(w.q_lens.max()) if w.batch else 0
        self.max_kv = int(w.kv_lens.max()) if w.batch else 0
        self.max_k = int(w.keep.max()) if w.batch else 0
        self.total_k = w.total_k
        self.any_dense = bool((w.seq_mode == hcsa.DLLM_SEQ_DENSE).any())
        self.batch = hcsa.make_batch(self.q, self.k, self.v, self.cu_q, self.cu_kv, self.max_q, self.max_kv,
                                w.softmax_scale)
        self.idx = torch.zeros((w.n_q_heads, max(1, w.total_k)), dtype=torch.int32, device=self.device)[:, :w.total_k]
        self.o = torch.zeros_like(self.q)

    def select(self, pool_w: int = 1, workspace=None):
        return hcsa.dllm_hcsa_select(self.batch, self.cu_k, self.total_k, self.max_k, self.idx, pool_w, workspace)

    def select_ex(self, pool_w: int = 1, forced_tail: int = 0, head_sum: bool = False, workspace=None):
        return hcsa.dllm_hcsa_select_ex(self.batch, self.cu_k, self.total_k, self.max_k, self.idx, pool_w, forced_tail,
                                   head_sum, workspace)

    def attend(self, idx=None, workspace=None):
        return hcsa.dllm_hcsa_attend(self.batch, self.idx if idx is None else idx, self.cu_k, self.total_k, self.max_k,
                                self.seq_mode if self.any_dense else None, self.o, workspace)

    def dense_refresh(self):
        return hcsa.dllm_dense_refresh_attend(self.batch, self.o)

    def pack(self, idx=None):
        """Pack the kept rows (allocates the packed buffers and their batch descriptor once)."""
        if not hasattr(self, "k_packed"):
            shape = (self.w.n_q_heads, self.total_k, self.w.head_dim)
            self.k_packed = torch.empty(shape, dtype=self.q.dtype, device=self.device)
            self.v_packed = torch.empty(shape, dtype=self.q.dtype, device=self.device)
            self.packed_batch = hcsa.make_packed_batch(self.q, self.k_packed, self.v_packed, self.cu_q, self.cu_k,
                                                  self.max_q, self.max_k, self.w.softmax_scale)
        return hcsa.dllm_hcsa_pack(self.batch, self.idx if idx is None else idx, self.cu_k, self.total_k, self.max_k,
                              self.k_packed, self.v_packed)

    def attend_packed(self, workspace=None):
        """Reuse attention over the packed cache: identity lists (idx = NULL) on the packed batch."""
        return hcsa.dllm_hcsa_attend(self.packed_batch, None, self.cu_k, self.total_k, self.max_k, None, self.o, workspace)
