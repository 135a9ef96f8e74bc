"""Device-memory plumbing around the C ABI: PyTorch is used only to own HBM buffers and streams.

DraftTrainer uploads a host workload (numpy) once, keeps params / grads / Adam state / workspace
resident, and forwards each call to the library.  It performs no arithmetic of the method.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from . import workloads as W


def _np_to_dev(x, dtype, device):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16" and t.dtype == torch.float32:
        # values are already bf16-representable (workloads.round_to_bf16): the cast is exact
        return t.to(device).to(torch.bfloat16)
    return t.to(device)


class DraftTrainer:
    def __init__(self, cfg: dict, params: dict, device="cuda:0"):
        self.cfg = dict(cfg)
        self.device = torch.device(device)
        self.dtype = cfg["dtype"]
        self.ccfg = B.make_config(cfg)
        dt = self.dtype
        self.params = {k: _np_to_dev(np.asarray(v, np.float32), dt, self.device) for k, v in params.items()}
        f32 = dict(dtype=torch.float32, device=self.device)
        self.grads = {k: torch.zeros(v.shape, **f32) for k, v in self.params.items()}
        self.m = {k: torch.zeros(v.shape, **f32) for k, v in self.params.items()}
        self.v = {k: torch.zeros(v.shape, **f32) for k, v in self.params.items()}
        self.master = ({k: v.to(torch.float32) for k, v in self.params.items()} if dt == "bf16" else None)
        self.ws_bytes = B.tide_draft_workspace_bytes(self.ccfg)
        if self.ws_bytes == 0:
            raise B.TideError(B.TIDE_ERR_CONFIG, B.tide_last_error())
        self.workspace = torch.empty(self.ws_bytes, dtype=torch.uint8, device=self.device)
        assert self.workspace.data_ptr() % 256 == 0
        self.loss = torch.zeros(1, **f32)
        self.c_params = B.make_tensors(self.params)
        self.c_grads = B.make_tensors(self.grads)
        self.c_adam = B.TideAdamState()
        self.c_adam.m = B.make_tensors(self.m)
        self.c_adam.v = B.make_tensors(self.v)
        self.c_adam.master = B.make_tensors(self.master)
        self.c_adam.step = 0
        self.hidden = self.tokens = self.mask = None

    # ---- inputs ----
    def set_batch(self, hidden, tokens, mask):
        """numpy (host) or torch (device) inputs; kept resident."""
        if isinstance(hidden, np.ndarray):
            hidden = _np_to_dev(hidden.astype(np.float32, copy=False), self.dtype, self.device)
        if isinstance(tokens, np.ndarray):
            tokens = torch.from_numpy(np.ascontiguousarray(tokens, dtype=np.int32)).to(self.device)
        if isinstance(mask, np.ndarray):
            mask = torch.from_numpy(np.ascontiguousarray(mask, dtype=np.uint8)).to(self.device)
        self.hidden, self.tokens, self.mask = hidden.contiguous(), tokens.contiguous(), mask.contiguous()

    def _stream(self):
        return torch.cuda.current_stream(self.device).cuda_stream

    # ---- calls ----
    def forward(self, want_top1=False):
        top1 = (torch.empty(self.cfg["batch"] * self.cfg["seq"], dtype=torch.int32, device=self.device)
                if want_top1 else None)
        B.tide_draft_forward(self.ccfg, self.c_params, self.hidden, self.tokens, self.mask, self.loss, top1,
                             self.workspace, self.ws_bytes, self._stream())
        return (self.loss, top1) if want_top1 else self.loss

    def eval(self):
        """(loss, top-1 accuracy over the loss-carrying positions), device scalars."""
        acc = torch.zeros(1, dtype=torch.float32, device=self.device)
        B.tide_draft_eval(self.ccfg, self.c_params, self.hidden, self.tokens, self.mask, self.loss, acc,
                          self.workspace, self.ws_bytes, self._stream())
        return self.loss, acc

    # ---- packed (variable-length) batches: the batch*seq rows hold sequences back to back ----
    def set_packed(self, cu_seqlens, max_seqlen=None):
        """cu_seqlens: n_seqs+1 ascending offsets into the rows (host list / numpy); kept resident on the device."""
        cu = np.ascontiguousarray(np.asarray(cu_seqlens, dtype=np.int32))
        self.n_seqs = int(cu.shape[0] - 1)
        self.max_seqlen = int(max_seqlen if max_seqlen is not None else max(1, int(np.max(np.diff(cu))) if self.n_seqs else 1))
        self.cu = torch.from_numpy(cu).to(self.device)

    def forward_packed(self, want_top1=False):
        top1 = (torch.empty(self.cfg["batch"] * self.cfg["seq"], dtype=torch.int32, device=self.device)
                if want_top1 else None)
        B.tide_draft_forward_packed(self.ccfg, self.c_params, self.hidden, self.tokens, self.mask, self.cu, self.n_seqs,
                                    self.max_seqlen, self.loss, top1, self.workspace, self.ws_bytes, self._stream())
        return (self.loss, top1) if want_top1 else self.loss

    def train_step_packed(self, lr):
        B.tide_draft_train_step_packed(self.ccfg, self.c_params, self.c_grads, self.c_adam, self.hidden, self.tokens,
                                       self.mask, self.cu, self.n_seqs, self.max_seqlen, lr, self.loss,
                                       self.workspace, self.ws_bytes, self._stream())
        return self.loss

    # ---- token-input variant: features joined with the sampled token's embedding through W_in ----
    def set_token_input(self, embed, input_ids, w_in):
        """numpy (host) arrays: embed [rows, d] (frozen), input_ids [B, S], w_in [d, 2d] (trainable); kept resident
        together with W_in's gradient and Adam state."""
        f32 = dict(dtype=torch.float32, device=self.device)
        self.embed = _np_to_dev(np.asarray(embed, np.float32), self.dtype, self.device)
        self.input_ids = torch.from_numpy(np.ascontiguousarray(input_ids, dtype=np.int32)).to(self.device)
        self.w_in = _np_to_dev(np.asarray(w_in, np.float32), self.dtype, self.device)
        self.grad_w_in = torch.zeros(self.w_in.shape, **f32)
        self.m_w_in = torch.zeros(self.w_in.shape, **f32)
        self.v_w_in = torch.zeros(self.w_in.shape, **f32)
        self.master_w_in = self.w_in.to(torch.float32) if self.dtype == "bf16" else None
        self.c_tok = B.make_token_input(self.embed, self.input_ids, self.w_in, self.grad_w_in, self.m_w_in,
                                        self.v_w_in, self.master_w_in)

    def forward_tok(self, want_top1=False):
        top1 = (torch.empty(self.cfg["batch"] * self.cfg["seq"], dtype=torch.int32, device=self.device)
                if want_top1 else None)
        B.tide_draft_forward_tok(self.ccfg, self.c_params, self.c_tok, self.hidden, self.tokens, self.mask, self.loss,
                                 top1, self.workspace, self.ws_bytes, self._stream())
        return (self.loss, top1) if want_top1 else self.loss

    def train_step_tok(self, lr):
        B.tide_draft_train_step_tok(self.ccfg, self.c_params, self.c_grads, self.c_adam, self.c_tok, self.hidden,
                                    self.tokens, self.mask, lr, self.loss, self.workspace, self.ws_bytes, self._stream())
        return self.loss

    # ---- multi-step unroll: the draft fed its own output from the second step on ----
    def _unroll_workspace(self, n_steps):
        need = B.tide_draft_unroll_workspace_bytes(self.ccfg, n_steps)
        if need == 0:
            raise B.TideError(B.TIDE_ERR_CONFIG, B.tide_last_error())
        if getattr(self, "unroll_ws", None) is None or self.unroll_ws.numel() < need:
            self.unroll_ws = torch.empty(need, dtype=torch.uint8, device=self.device)

    def train_step_unroll(self, lr, n_steps, step_weights=None, token_input=False, packed=False):
        """One AdamW step on sum_s step_weights[s] * loss_s; returns the per-step losses (device vector).
        packed: the batch is the packed one of set_packed."""
        self._unroll_workspace(n_steps)
        loss = torch.zeros(n_steps, dtype=torch.float32, device=self.device)
        tok = self.c_tok if token_input else None
        if packed:
            B.tide_draft_train_step_unroll_packed(self.ccfg, self.c_params, self.c_grads, self.c_adam, tok, self.hidden,
                                                  self.tokens, self.mask, self.cu, self.n_seqs, self.max_seqlen, n_steps,
                                                  step_weights, lr, loss, self.unroll_ws, self.unroll_ws.numel(), self._stream())
        else:
            B.tide_draft_train_step_unroll(self.ccfg, self.c_params, self.c_grads, self.c_adam, tok, self.hidden, self.tokens,
                                           self.mask, n_steps, step_weights, lr, loss, self.unroll_ws, self.unroll_ws.numel(),
                                           self._stream())
        return loss

    def eval_unroll(self, n_steps, token_input=False, packed=False):
        """(loss [n_steps], accuracy [n_steps]) device vectors; the unroll keeps a workspace of its own."""
        self._unroll_workspace(n_steps)
        loss = torch.zeros(n_steps, dtype=torch.float32, device=self.device)
        acc = torch.zeros(n_steps, dtype=torch.float32, device=self.device)
        tok = self.c_tok if token_input else None
        if packed:
            B.tide_draft_eval_unroll_packed(self.ccfg, self.c_params, tok, self.hidden, self.tokens, self.mask, self.cu,
                                            self.n_seqs, self.max_seqlen, n_steps, loss, acc, self.unroll_ws,
                                            self.unroll_ws.numel(), self._stream())
        else:
            B.tide_draft_eval_unroll(self.ccfg, self.c_params, tok, self.hidden, self.tokens, self.mask, n_steps, loss, acc,
                                     self.unroll_ws, self.unroll_ws.numel(), self._stream())
        return loss, acc

    def train_step(self, lr):
        B.tide_draft_train_step(self.ccfg, self.c_params, self.c_grads, self.c_adam, self.hidden, self.tokens,
                                self.mask, lr, self.loss, self.workspace, self.ws_bytes, self._stream())
        return self.loss

    def train_step_dev(self, lr_dev, step_dev):
        """The training step with its learning rate (device float) and step count (device int64) in device memory:
        capturable into a HIP graph; the count is advanced on the device."""
        B.tide_draft_train_step_dev(self.ccfg, self.c_params, self.c_grads, self.c_adam, self.hidden, self.tokens,
                                    self.mask, lr_dev, step_dev, self.loss, self.workspace, self.ws_bytes, self._stream())
        return self.loss

    def status(self):
        """Device status word of the last call (0 = fine, 1 = loss not finite, 2 = malformed cu_seqlens); synchronises."""
        off = B.tide_draft_workspace_offset(self.ccfg, "status")
        return int(self.workspace[off:off + 4].view(torch.int32).item())

    @property
    def step(self):
        return int(self.c_adam.step)

    # ---- read-back helpers for tests ----
    def intermediate(self, name, shape, kind="act"):
        """View of a named workspace buffer; kind: 'act' (config dtype) or 'f32'."""
        off = B.tide_draft_workspace_offset(self.ccfg, name)
        if off < 0:
            raise KeyError(name)
        tdt = torch.float32 if (kind == "f32" or self.dtype == "fp32") else torch.bfloat16
        n = int(np.prod(shape))
        nbytes = n * (4 if tdt == torch.float32 else 2)
        return self.workspace[off:off + nbytes].view(tdt).view(*shape)

    def host(self, d):
        return {k: v.detach().to(torch.float32).cpu().numpy().astype(np.float64) for k, v in d.items()}


def trainer_from_workload(cfg, wl, device="cuda:0"):
    tr = DraftTrainer(cfg, wl["params"], device=device)
    tr.set_batch(wl["hidden"], wl["tokens"], wl["mask"])
    return tr
