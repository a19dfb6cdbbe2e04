"""Device-memory plumbing around the C ABI for tests, the smoke check and the
benchmark: owns torch tensors (weights, KV caches, workspace, I/O vectors) and
forwards to the library.  No arithmetic of the decode path happens here."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B


class DeviceStack:
    """An L-layer stack resident on one GPU (L = 1 for a single block)."""

    def __init__(self, shape, max_seq: int, max_batch: int = 1, n_layers: int | None = None,
                 device: str = "cuda:0", share_weights_of: "DeviceStack | None" = None):
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the HIP path has no CPU fallback")
        self.shape = shape
        self.dev = torch.device(device)
        torch.cuda.set_device(self.dev)
        self.L = shape.n_layers if n_layers is None else n_layers
        self.cfg = B.Config.from_shape(shape, max_seq, max_batch, self.L)
        st = B.cfpp_validate_config(self.cfg)
        if st != 0:
            raise B.CfppError(st, "cfpp_validate_config", B.lib().cfpp_last_error().decode())
        self.max_seq, self.max_batch = max_seq, max_batch
        u8 = dict(dtype=torch.uint8, device=self.dev)
        # (packed layers do not depend on max_seq or max_batch: another stack's can be borrowed)
        self.packed = (share_weights_of.packed[: self.L] if share_weights_of is not None else
                       [torch.empty(B.cfpp_packed_layer_bytes(self.cfg), **u8) for _ in range(self.L)])
        # 0xFF bytes = fp16 NaN everywhere: any read of a never-written slot shows up
        self.kv = [torch.full((B.cfpp_kv_layer_bytes(self.cfg),), 0xFF, **u8) for _ in range(self.L)]
        self.ws_bytes = B.cfpp_workspace_bytes(self.cfg)
        self.ws = torch.empty(self.ws_bytes, **u8)
        self.x = torch.zeros(max_batch, shape.hidden, dtype=torch.float16, device=self.dev)
        self.out = torch.zeros_like(self.x)
        self.pos = torch.zeros(max_batch, dtype=torch.int32, device=self.dev)
        self.stream = torch.cuda.Stream(device=self.dev)
        torch.cuda.synchronize()
        self.ctx = B.cfpp_create(self.cfg, self.ws, self.ws_bytes)

    def close(self):
        if self.ctx:
            torch.cuda.synchronize()
            B.cfpp_destroy(self.ctx)
            self.ctx = 0

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- options ---------------------------------------------------------
    def set_options(self, mode=None, grid=None, threads=None):
        if mode is not None:
            B.cfpp_set_option(self.ctx, B.OPT_MODE, mode)
        if grid is not None:
            B.cfpp_set_option(self.ctx, B.OPT_GRID, grid)
        if threads is not None:
            B.cfpp_set_option(self.ctx, B.OPT_THREADS, threads)

    @property
    def s(self) -> int:
        return self.stream.cuda_stream

    # -- data ------------------------------------------------------------
    def load_layer(self, l: int, w: dict):
        """w: canonical fp16 numpy tensors of one block."""
        dev = {n: torch.from_numpy(np.ascontiguousarray(w[n])).to(self.dev) for n in B.LAYER_TENSORS}
        torch.cuda.synchronize()
        B.cfpp_pack_layer(self.cfg, dev, self.packed[l], self.s)
        self.stream.synchronize()

    def load_layer_device(self, l: int, dev_tensors: dict):
        """dev_tensors: canonical fp16 torch tensors of one block, already on this GPU."""
        torch.cuda.synchronize()
        B.cfpp_pack_layer(self.cfg, dev_tensors, self.packed[l], self.s)
        self.stream.synchronize()

    def load_kv(self, l: int, K: np.ndarray, V: np.ndarray, n_cached):
        """K, V: fp16 [batch, n_heads, capacity, head_dim]; the first n_cached[b]
        positions of each sequence are imported."""
        n_cached = np.broadcast_to(np.asarray(n_cached), (K.shape[0],))
        for b in range(K.shape[0]):
            k = torch.from_numpy(np.ascontiguousarray(K[b])).to(self.dev)
            v = torch.from_numpy(np.ascontiguousarray(V[b])).to(self.dev)
            torch.cuda.synchronize()
            B.cfpp_kv_import(self.cfg, k, v, K.shape[2], int(n_cached[b]), b, self.kv[l], self.s)
            self.stream.synchronize()

    def export_kv(self, l: int, b: int, pos_begin: int, n_pos: int):
        H, d = self.shape.n_heads, self.shape.head_dim
        k = torch.zeros(H, n_pos, d, dtype=torch.float16, device=self.dev)
        v = torch.zeros_like(k)
        torch.cuda.synchronize()
        B.cfpp_kv_export(self.cfg, self.kv[l], b, pos_begin, n_pos, n_pos, k, v, self.s)
        self.stream.synchronize()
        return k.cpu().numpy(), v.cpu().numpy()

    def set_inputs(self, x: np.ndarray, pos):
        x = np.asarray(x, dtype=np.float16).reshape(-1, self.shape.hidden)
        self.batch = x.shape[0]
        self.x[: self.batch].copy_(torch.from_numpy(x))
        p = np.broadcast_to(np.asarray(pos, dtype=np.int32), (self.batch,)).copy()
        self.pos[: self.batch].copy_(torch.from_numpy(p))
        torch.cuda.synchronize()

    def result(self) -> np.ndarray:
        self.stream.synchronize()
        return self.out[: self.batch].cpu().numpy()

    # -- hot path --------------------------------------------------------
    def block_decode(self, l: int = 0):
        B.cfpp_block_decode(self.ctx, self.packed[l], self.kv[l], self.x, self.pos, self.batch,
                            self.out, self.s)

    def stack_decode(self):
        B.cfpp_stack_decode(self.ctx, self.packed, self.kv, self.x, self.pos, self.batch, self.out, self.s)

    def prefill(self, x: np.ndarray, pos0: int, b: int = 0) -> np.ndarray:
        """x: fp16 [T, hidden] prompt rows, appended to sequence b from position pos0 on;
        returns the last block's fp16 output per token."""
        xd = torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)
        od = torch.zeros_like(xd)
        torch.cuda.synchronize()
        B.cfpp_stack_prefill(self.ctx, self.packed, self.kv, xd, pos0, x.shape[0], b, od, self.s)
        self.stream.synchronize()
        return od.cpu().numpy()

    def prefill_gemm(self, x: np.ndarray, pos0: int, b: int = 0, rows: int = 128) -> np.ndarray:
        """As prefill(), through the prompt-sized kernels, `rows` tokens per pass."""
        xd = torch.from_numpy(np.ascontiguousarray(x)).to(self.dev)
        od = torch.zeros_like(xd)
        nbytes = B.cfpp_prefill_scratch_bytes(self.cfg, rows)
        if nbytes == 0:
            raise B.CfppError(-1, "cfpp_prefill_scratch_bytes", "invalid configuration or rows")
        scratch = torch.empty(nbytes, dtype=torch.uint8, device=self.dev)
        torch.cuda.synchronize()
        B.cfpp_stack_prefill_gemm(self.ctx, self.packed, self.kv, xd, pos0, x.shape[0], b, od, scratch, nbytes, rows, self.s)
        self.stream.synchronize()
        return od.cpu().numpy()

    def capture(self):
        B.cfpp_stack_capture(self.ctx, self.packed, self.kv, self.x, self.pos, self.batch, self.out, self.s)

    def replay(self):
        B.cfpp_stack_replay(self.ctx, self.s)

    # -- generation loop ---------------------------------------------------
    def load_lm(self, head: dict, embed: np.ndarray):
        """head: final LayerNorm + LM head (fp16 numpy: lnf_g, lnf_b, w_lm); embed: [vocab, hidden]."""
        self.vocab = int(head["w_lm"].shape[0])
        self.lm_t = {n: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
                     for n, a in (("embed", embed), ("lnf_g", head["lnf_g"]), ("lnf_b", head["lnf_b"]),
                                  ("w_lm", head["w_lm"]))}
        self.lm = B.Lm.of(self.lm_t["embed"], self.lm_t["lnf_g"], self.lm_t["lnf_b"], self.lm_t["w_lm"], self.vocab)
        self.tokens = torch.zeros(self.max_seq + 1, dtype=torch.int32, device=self.dev)
        self.logits = torch.zeros(self.vocab, dtype=torch.float32, device=self.dev)
        self.batch = 1
        torch.cuda.synchronize()

    def set_tokens(self, tokens, pos: int):
        """tokens[0..pos] are known; generation continues from position pos."""
        t = np.zeros(self.max_seq + 1, dtype=np.int32)
        t[: pos + 1] = np.asarray(tokens[: pos + 1], dtype=np.int32)
        self.tokens.copy_(torch.from_numpy(t))
        self.pos[:1].copy_(torch.tensor([pos], dtype=torch.int32))
        torch.cuda.synchronize()

    def generate_step(self, want_logits: bool = False):
        """One token, call by call (no graph): embed, stack, next token."""
        B.cfpp_lm_embed(self.ctx, self.lm, self.tokens, self.pos, self.x, self.s)
        B.cfpp_stack_decode(self.ctx, self.packed, self.kv, self.x, self.pos, 1, self.out, self.s)
        B.cfpp_lm_next(self.ctx, self.lm, self.out, self.tokens, self.pos,
                       self.logits if want_logits else None, self.s)

    def generate_capture(self):
        B.cfpp_generate_capture(self.ctx, self.packed, self.kv, self.lm, self.tokens, self.pos, self.x,
                                self.out, self.s)

    def check(self):
        B.cfpp_device_error(self.ctx, self.s)

    def tap(self, which: int, count: int) -> np.ndarray:
        return B.cfpp_debug_read(self.ctx, which, count, self.s)
