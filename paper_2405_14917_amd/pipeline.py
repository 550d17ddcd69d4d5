"""Drivers above the binding: the order of the entry points for one linear layer (Alg. 1), and for several
layers that read the same input (q/k/v or gate/up of a transformer block), which need ONE Hessian and ONE inverse
between them because H = 2 X X^T belongs to the input, not to the layer (Eq. 3).

Only sequencing happens here: every step runs in the library's kernels.  Buffers that do not depend on the
layer (G, U, diag H^-1) are allocated once per driver."""
import torch

from . import binding


class LayerPass:
    """The hot path over resident layers with m input channels.

    Two library contexts on two streams: the half of the bit allocation that needs neither the Hessian nor the
    salience (the reference outputs and the outputs of the all-N-bit weights, two n x m x t_s products) is enqueued
    on the second stream before the inverse, whose chain of small kernels leaves most of the chip idle."""

    def __init__(self, slim, m, beta, N, percdamp=0.01, t_sba=2048, device="cuda:0", n=None):
        """n (output rows of the largest layer that will be passed): if given, the second context gets a workspace of
        the size slim_workspace_query states for the bit allocation of such a layer, allocated here once, so that no
        call on it allocates; without it the context grows its own."""
        self.slim, self.m, self.beta, self.N, self.percdamp, self.t_sba = slim, m, beta, N, percdamp, t_sba
        self.bit_base = binding.bit_base_for(N)     # of the stored form: what its 2-bit group value 0 stands for
        self.G = torch.zeros((m, m), dtype=torch.float32, device=device)
        self.U = torch.empty((m, m), dtype=torch.float64, device=device)
        self.d = torch.empty(m, dtype=torch.float64, device=device)
        self.main = torch.cuda.current_stream()
        self.side = torch.cuda.Stream()
        with torch.cuda.stream(self.side):
            self.slim_sba = binding.Slim(device, 0 if n is None else binding.workspace_query(n, m, beta, 0, t_sba))

    def contexts(self):
        return [self.slim, self.slim_sba]

    def close(self):
        self.slim_sba.close()

    def _hessian_and_first_prepare(self, W, X):
        """G = X X^T, then the damped inverse with the rank-independent half of W's bit allocation beside it."""
        s, s2 = self.slim, self.slim_sba
        Xs = X[:, : min(self.t_sba, X.shape[1])]
        self.G.zero_()
        nt = s.hessian_accumulate(X, self.G, 0)
        self.side.wait_stream(self.main)               # the Gram kernel has the chip to itself
        s2.sba_prepare(W, self.beta, self.N, Xs)
        s.hessian_inverse(self.G, nt, self.percdamp, U=self.U, hinv_diag=self.d)
        return Xs

    def _allocate_quantize_pack(self, W, Xs, prepared):
        """Salience, bit allocation (on the second context when its first half is already there), sweep, packing."""
        s, s2 = self.slim, self.slim_sba
        _, grp, _ = s.salience(W, self.d, self.beta)
        # no call here asks for a host output (p_star and m_star stay on the device).  The one wait of the host
        # inside a pass is the sweep's: it reads the k widths back, for validation and to choose its kernels, behind
        # the widening of W that it has already enqueued
        if prepared:
            self.side.wait_stream(self.main)
            with torch.cuda.stream(self.side):
                bits, _, _ = s2.sba_allocate(W, grp, self.beta, self.N, Xs, host_outputs=False)
            grp.record_stream(self.side)
            bits.record_stream(self.main)
            self.main.wait_stream(self.side)
        else:
            bits, _, _ = s.sba_allocate(W, grp, self.beta, self.N, Xs, host_outputs=False)
        out = s.gptq_quantize(W, self.U, bits, self.beta)
        packed, gbits, row_off, _ = s.pack(out["codes"], bits, self.beta, packed_rows=self.m * (self.N + 1) // 32,
                                           host_outputs=False, bit_base=self.bit_base)
        return {"bits": bits, "bit_base": self.bit_base, "p_star": (bits == self.N - 1).sum(), "codes": out["codes"],
                "scale": out["scale"],
                "zero": out["zero"], "packed": packed, "gbits": gbits, "row_off": row_off, "m_star": row_off[-1]}

    def run(self, W, X):
        """One layer: W (n x m), X (m x t, fp16 / bf16, tokens contiguous).  Returns device tensors only (p_star and
        m_star as 0-dim tensors; packed with the rows of its capacity, zero from row m_star on)."""
        Xs = self._hessian_and_first_prepare(W, X)
        return self._allocate_quantize_pack(W, Xs, True)

    def run_shared_input(self, Ws, X):
        """Layers that read the same input: one Hessian and one inverse, then each layer's own steps.  The result
        of every layer is the one `run` gives for it alone."""
        Xs = self._hessian_and_first_prepare(Ws[0], X)
        return [self._allocate_quantize_pack(W, Xs, i == 0) for i, W in enumerate(Ws)]
