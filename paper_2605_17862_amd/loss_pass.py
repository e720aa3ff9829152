"""Convenience holder of the output and workspace buffers of one problem size.

Only allocation and argument plumbing: each method is one call of the binding.
"""

import torch

from . import binding as fb

DEFAULT_HPARAMS = (1.0, 1.0, 0.05, 0.1)     # alpha, beta, xi, lambda (not values from the paper)


class LossPass:
    def __init__(self, T, V, B, dtype, ld=None, device="cuda:0", alloc_dlogits=True):
        self.T, self.V, self.B = int(T), int(V), int(B)
        self.ld = self.V if ld is None else int(ld)
        self.dt = fb.FOPD_BF16 if dtype in ("bf16", torch.bfloat16) else fb.FOPD_F32
        self.torch_dtype = torch.bfloat16 if self.dt == fb.FOPD_BF16 else torch.float32
        dev = torch.device(device)
        f32 = dict(dtype=torch.float32, device=dev)
        self.logp = torch.empty(self.T, **f32)
        self.lse = torch.empty(self.T, **f32)
        self.gather_idx = torch.empty(self.T, dtype=torch.int64, device=dev)
        self.entropy = None
        self.cu_seqlens = torch.empty(self.B + 1, dtype=torch.int64, device=dev)
        self.n_train = torch.empty(self.B, dtype=torch.int32, device=dev)
        self.n_roll = torch.empty(self.B, dtype=torch.int32, device=dev)
        self.D_roll = torch.empty(self.B, **f32)
        self.D_sup = torch.empty(self.B, **f32)
        self.ell = torch.empty(self.B, **f32)
        self.cover = torch.empty(self.B, **f32)
        self.cover_roll = torch.empty(self.B, **f32)
        self.freshness = torch.empty(self.B, **f32)
        self.weights = torch.empty(self.B, **f32)
        self.agg = torch.empty(3, **f32)
        self.loss = torch.empty(1, **f32)
        self.dlogits = (torch.empty(self.T, self.ld, dtype=self.torch_dtype, device=dev)
                        if alloc_dlogits else None)
        nbytes = fb.fopd_workspace_bytes(self.T, self.B)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=dev)
        off = (-self.workspace.data_ptr()) % 256
        self.workspace = self.workspace[off:off + nbytes]
        fb.fopd_workspace_init(self.workspace)

    def token_logprobs(self, w, rows=None, want_gather=True, want_entropy=False):
        a, b = (0, self.T) if rows is None else rows
        if want_entropy and self.entropy is None:
            self.entropy = torch.empty(self.T, dtype=torch.float32, device=self.logp.device)
        fb.fopd_token_logprobs(w["logits"][a:b], self.dt, b - a, self.V, self.ld, w["token_ids"][a:b],
                               w["mask"][a:b], self.logp[a:b], self.lse[a:b],
                               self.gather_idx[a:b] if want_gather else None,
                               self.entropy[a:b] if want_entropy else None, self.workspace)

    def freshness_score(self, w, hp=DEFAULT_HPARAMS):
        stale = w["teacher_logp_stale"]
        fb.fopd_freshness_score(self.logp, w["behav_logp"], None, None, w["teacher_logp"], stale, w["mask"],
                                w["seq_lens"], w["lag"], self.T, self.B, hp, self.cu_seqlens, self.n_train,
                                self.n_roll, self.D_roll, self.D_sup, self.ell, self.cover, self.cover_roll,
                                self.freshness, self.agg, self.workspace)

    def loss_fwd_bwd(self, w, hp=DEFAULT_HPARAMS, grad_scale=1.0, dlogits=None):
        """Everything in one call: scores, weights, loss and gradient."""
        out = self.dlogits if dlogits is None else dlogits
        fb.fopd_loss_fwd_bwd(w["logits"], self.dt, self.T, self.V, self.ld, w["token_ids"], w["mask"],
                             w["behav_logp"], w["teacher_logp"], w["teacher_logp_stale"], w["seq_lens"],
                             w["lag"], self.B, hp, None, None, None, 0, None, None, grad_scale, self.loss,
                             self.freshness, self.weights, self.logp, out, self.workspace)

    def status(self):
        return fb.fopd_workspace_status(self.workspace)
