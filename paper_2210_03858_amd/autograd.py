"""torch.autograd front end of the BCQ linear layer (AlphaTuning Section 4.1: the sign planes are frozen, only the
scales are trained; Section 4.2: normally alpha_1 alone).

`BCQLinearFunction` routes forward (Eq. 2), input gradient (Eq. 3) and scale gradient (Eq. 4) to the C-ABI entry
points; `BCQLinear` is the module around it.  Nothing is computed here: every product runs in the HIP kernels.
"""
import torch

from . import binding as B


class _Layer:
    """Frozen state of one quantized layer: packed planes, optional transposed twin, workspaces by token count."""

    def __init__(self, packed, g, q_train, grad_scale, twin=True):
        self.packed = packed
        self.q, self.N, kw = packed.shape
        self.K = kw * 32
        self.g = self.K if g is None else int(g)
        self.q_train = self.q if q_train is None else int(q_train)
        self.grad_scale = float(grad_scale)
        self.twin = B.bcq_pack_transposed(packed) if (twin and self.N % 32 == 0) else None
        self._ws = {}

    def workspace(self, op, T, dtype_code):
        key = (op, T, dtype_code)
        if key not in self._ws:
            n = B.workspace_bytes_grouped(op, T, self.N, self.K, self.g, self.q, dtype_code)
            self._ws[key] = torch.empty((max(n, 16),), dtype=torch.uint8, device=self.packed.device)
        return self._ws[key]


class BCQLinearFunction(torch.autograd.Function):
    @staticmethod
    def forward(ctx, x, alpha_train, alpha_frozen, layer):
        alpha = alpha_train if alpha_frozen is None else torch.cat((alpha_train, alpha_frozen), dim=0)
        alpha = alpha.contiguous()
        x2 = x.reshape(-1, layer.K).contiguous()
        code = B._act_dtype(x2)
        y = B.bcq_linear_fwd_grouped(layer.packed, alpha, x2, layer.g,
                                     workspace=layer.workspace(B.OP_FWD, x2.shape[0], code))
        ctx.layer = layer
        ctx.save_for_backward(x2, alpha)
        ctx.x_shape = x.shape
        return y.reshape(*x.shape[:-1], layer.N)

    @staticmethod
    def backward(ctx, dy):
        layer = ctx.layer
        x2, alpha = ctx.saved_tensors
        dy2 = dy.reshape(-1, layer.N).contiguous()
        code = B._act_dtype(dy2)
        T = dy2.shape[0]
        dx = da = None
        if ctx.needs_input_grad[0]:
            dx = B.bcq_linear_bwd_input_grouped(layer.packed, alpha, dy2, layer.g, packed_t=layer.twin,
                                                workspace=layer.workspace(B.OP_BWD_INPUT, T, code)).reshape(ctx.x_shape)
        if ctx.needs_input_grad[1]:
            da = B.bcq_linear_bwd_alpha_grouped(layer.packed, x2, dy2, layer.g, q_train=layer.q_train,
                                                grad_scale=layer.grad_scale,
                                                workspace=layer.workspace(B.OP_BWD_ALPHA, T, code))
        return dx, da, None, None


class BCQLinear(torch.nn.Module):
    """y = x What^T (+ bias), What = sum_i diag(alpha_i) B_i with frozen packed sign planes.

    alpha[:q_train] is the trainable parameter `alpha_train` ([q_train, N, K/g] fp32); the other planes' scales and
    the bias are frozen buffers (Section 4.2).  grad_scale multiplies the scale gradient: 1 gives the true gradient,
    1/g is the damping of Eq. 4."""

    def __init__(self, packed, alpha, g=None, bias=None, q_train=1, grad_scale=1.0):
        super().__init__()
        q, N, kw = packed.shape
        K = kw * 32
        g = K if g is None else int(g)
        alpha = alpha.reshape(q, N, K // g).to(torch.float32).contiguous()
        self.register_buffer("packed", packed)
        self.alpha_train = torch.nn.Parameter(alpha[:q_train].clone())
        self.register_buffer("alpha_frozen", alpha[q_train:].clone() if q_train < q else None)
        self.register_buffer("bias", bias)
        self._layer = _Layer(packed, g, q_train, grad_scale)

    @classmethod
    def from_weight(cls, W, q, g=None, bias=None, q_train=1, grad_scale=1.0, alternating_iters=None):
        """Quantize a dense fp32 weight [N, K] on the GPU: greedy (Appendix C), or alternating with the given rounds."""
        K = W.shape[1]
        g = K if g is None else int(g)
        if alternating_iters is None:
            alpha, packed, _ = B.bcq_quantize_grouped(W.contiguous(), q, g)
        else:
            alpha, packed, _ = B.bcq_quantize_alternating(W.contiguous(), q, iters=alternating_iters, g=g)
        return cls(packed, alpha, g=g, bias=bias, q_train=q_train, grad_scale=grad_scale)

    def forward(self, x):
        y = BCQLinearFunction.apply(x, self.alpha_train, self.alpha_frozen, self._layer)
        return y if self.bias is None else y + self.bias.to(y.dtype)
