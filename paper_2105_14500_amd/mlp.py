"""One processor's share of the Tesseract MLP (Section 3.2.1: two linear layers with an
activation in the middle), as a chain of library calls on one stream.

Sequencing only: every product, bias add, activation, activation gradient and bias
gradient runs inside the HIP library.  What a processor produces itself feeds panel
slot `own` of the next call (its own block column / block row); the other q-1 panels of
each operand are the blocks that the row and column broadcasts of Alg. 3 deliver, given
by the caller.

Shapes for a grid [q, q, d] with hidden size h, f = 4h, m rows per block:
  up:   X panels [m, h/q],  W1 panels [h/q, f/q], bias1 [f/q]  -> Z1, H = act(Z1)  [m, f/q]
  down: H panels [m, f/q],  W2 panels [f/q, h/q], bias2 [h/q]  -> Y               [m, h/q]
"""
import torch

from . import binding as B


class MlpShare:
    def __init__(self, q, d, m, h_q, f_q, act=B.ACT_GELU_ERF, own=0, device="cuda:0"):
        self.q, self.d, self.m, self.h_q, self.f_q, self.act, self.own = q, d, m, h_q, f_q, act, own
        a = m * q * d
        self.up = B.make_desc(q, d, 0, 0, 0, a, h_q * q, f_q * q, B.BF16, B.BF16)
        self.down = B.make_desc(q, d, 0, 0, 0, a, f_q * q, h_q * q, B.BF16, B.BF16)
        nbytes = max(B.workspace_bytes(dsc, op) for dsc in (self.up, self.down) for op in (0, 1, 2))
        self.ws = torch.empty(max(nbytes, 4) // 4, dtype=torch.float32, device=device)
        bf, f32 = torch.bfloat16, torch.float32
        new = lambda r, c, dt: torch.empty((r, c), dtype=dt, device=device)
        self.z1, self.h, self.y = new(m, f_q, bf), new(m, f_q, bf), new(m, h_q, bf)
        self.dz1, self.dx = new(m, f_q, bf), new(m, h_q, bf)
        self.dw1, self.dw2 = torch.zeros((h_q, f_q), dtype=f32, device=device), \
            torch.zeros((f_q, h_q), dtype=f32, device=device)
        self.db1, self.db2 = torch.zeros((f_q,), dtype=f32, device=device), \
            torch.zeros((h_q,), dtype=f32, device=device)

    def _with_own(self, panels, mine):
        p = list(panels)
        p[self.own] = mine
        return p

    def forward(self, x_panels, w1_panels, bias1, h_panels, w2_panels, bias2):
        """h_panels[own] is replaced by the block this processor computes."""
        B.linear_fwd(self.up, x_panels, w1_panels, bias1, self.act, self.h, preact_out=self.z1,
                     workspace=self.ws)
        B.linear_fwd(self.down, self._with_own(h_panels, self.h), w2_panels, bias2, B.ACT_NONE,
                     self.y, workspace=self.ws)
        return self.y

    def backward(self, x_panels, w1t_panels, h_panels, w2t_panels, dy_panels, dz1_panels,
                 accumulate=True):
        """dy_panels: gradient of the MLP output, blocks of this grid row (for dX) which here also
        stand for the blocks of this grid column (for dW).  w1t_panels / w2t_panels: block row
        `own` of W1 / W2 (what the dX products read).  dz1_panels[own] is replaced by the block
        this processor computes.  Weight and bias gradients live in fp32 buffers that the calls
        add to (the depth sum); with accumulate=False the buffers are cleared first."""
        if not accumulate:
            for t in (self.dw1, self.dw2, self.db1, self.db2):
                t.zero_()
        # down projection: weight + bias gradient, then input gradient through the activation
        B.linear_bwd_dw_bias(self.down, self._with_own(h_panels, self.h), dy_panels, self.dw2, self.db2,
                             accumulate=True, workspace=self.ws)
        B.linear_bwd_dx_act(self.down, dy_panels, w2t_panels, self.z1, self.act, self.dz1,
                            workspace=self.ws)
        # up projection
        dz = self._with_own(dz1_panels, self.dz1)
        B.linear_bwd_dw_bias(self.up, x_panels, dz, self.dw1, self.db1, accumulate=True,
                             workspace=self.ws)
        B.linear_bwd_dx(self.up, dz, w1t_panels, self.dx, workspace=self.ws)
        return self.dx

    def flops(self):
        """fwd + dX + dW of both layers: 6abc/p each."""
        return 2 * 3 * 2.0 * self.m * self.h_q * self.f_q * self.q
