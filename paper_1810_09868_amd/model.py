"""Buffer management around the model-level entry points (no arithmetic: all
compute happens in libvgg_mi355x.so).  torch is used only to own device
memory and the current stream."""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np
import torch

from . import binding as B

_CONV = [(3, 64), (64, 64), (64, 128), (128, 128), (128, 256), (256, 256), (256, 256), (256, 256),
         (256, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512), (512, 512)]


class Vgg19:
    """Owns the packed parameter block and the workspace for one configuration."""

    def __init__(self, dtype: int, N: int, H: int, W: int, fc_hidden: int, classes: int, lr: float = 0.01,
                 training: bool = False):
        if not torch.cuda.is_available():
            raise RuntimeError("Vgg19 needs a GPU: the HIP library is the only implementation")
        # bf16 training keeps fp32 master parameters behind the bf16 ones
        flags = B.FLAG_FP32_MASTER if (training and dtype == B.BF16) else 0
        self.cfg = B.make_config(dtype, N, H, W, fc_hidden, classes, lr, flags)
        self.training = training
        nb = B.vgg19_packed_bytes(self.cfg)
        if nb == 0:
            raise ValueError("invalid configuration")
        self.packed = torch.zeros((nb,), dtype=torch.uint8, device="cuda")
        wsb = B.vgg19_train_workspace_bytes(self.cfg) if training else B.vgg19_forward_workspace_bytes(self.cfg)
        if wsb == 0:
            raise ValueError("configuration not supported for this mode")
        # zeroed once: the update streams over the whole parameter block, alignment gaps included, and the
        # gaps of the gradient block inside the workspace are never written by a kernel
        self.ws = torch.zeros((wsb,), dtype=torch.uint8, device="cuda")
        self.logits = torch.empty((N, classes), dtype=torch.float32, device="cuda")
        self.probs = torch.empty((N, classes), dtype=torch.float32, device="cuda")
        self.loss = torch.zeros((1,), dtype=torch.float32, device="cuda")
        flat = 512 * (H // 32) * (W // 32)
        self.fc_dims = [(flat, fc_hidden), (fc_hidden, fc_hidden), (fc_hidden, classes)]

    # canonical fp32 device tensors for parameters / gradients
    def _canon_buffers(self) -> Dict[str, List[torch.Tensor]]:
        mk = lambda *s: torch.empty(s, dtype=torch.float32, device="cuda")
        return dict(conv_w=[mk(co, ci, 3, 3) for ci, co in _CONV], conv_b=[mk(co) for _, co in _CONV],
                    fc_w=[mk(o, i) for i, o in self.fc_dims], fc_b=[mk(o) for _, o in self.fc_dims])

    def pack(self, conv_w, conv_b, fc_w, fc_b) -> None:
        """Uploads canonical fp32 numpy parameters and packs them on the device."""
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
        t = dict(conv_w=[up(a) for a in conv_w], conv_b=[up(a) for a in conv_b],
                 fc_w=[up(a) for a in fc_w], fc_b=[up(a) for a in fc_b])
        B.vgg19_pack_params(self.cfg, B.make_params(**t), self.packed)
        torch.cuda.synchronize()

    def unpack(self) -> Dict[str, List[np.ndarray]]:
        t = self._canon_buffers()
        B.vgg19_unpack_params(self.cfg, self.packed, B.make_params(**t))
        torch.cuda.synchronize()
        return {k: [a.cpu().numpy() for a in v] for k, v in t.items()}

    def forward(self, x: torch.Tensor, want_probs: bool = True) -> None:
        B.vgg19_forward(self.cfg, x, self.packed, self.logits, self.probs if want_probs else None, self.ws)

    def train_step(self, x: torch.Tensor, labels: torch.Tensor, want_grads: bool = False
                   ) -> Optional[Dict[str, List[torch.Tensor]]]:
        if not self.training:
            raise RuntimeError("constructed with training=False")
        g = self._canon_buffers() if want_grads else None
        B.vgg19_train_step(self.cfg, x, labels, self.packed, B.make_params(**g) if g else None, self.loss,
                           self.logits, self.ws)
        return g

    def capture_forward(self, x: torch.Tensor, passes: int = 1, want_probs: bool = True) -> "torch.cuda.CUDAGraph":
        """Records `passes` forward passes on the given batch into one HIP graph (call forward once before
        capturing).  At small batches a pass is a few dozen short launches, and replaying them as one graph
        removes the host's share of the latency."""
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(passes):
                B.vgg19_forward(self.cfg, x, self.packed, self.logits, self.probs if want_probs else None, self.ws)
        return g

    def capture_train_steps(self, x: torch.Tensor, labels: torch.Tensor, steps: int) -> "torch.cuda.CUDAGraph":
        """Records `steps` consecutive training steps on the given batch into one HIP graph, so that the whole
        loop (forward, backward and update, `steps` times) is replayed by a single launch without returning to
        the host in between: the training loop itself runs on the device, as in the paper's whole-program
        compilation of "forward pass, backward pass and training loop" (introduction).  Call train_step once
        before capturing (first use of a kernel sets its LDS limit, which is not a stream operation).  The
        library records no memset nodes and allocates nothing, so every launch is capturable."""
        if not self.training:
            raise RuntimeError("constructed with training=False")
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(steps):
                B.vgg19_train_step(self.cfg, x, labels, self.packed, None, self.loss, self.logits, self.ws)
        return g

