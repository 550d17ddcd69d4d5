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

    def __init__(self, slim, m, beta, N, percdamp=0.01, t_sba=2048, device="cuda:0", n=None, second=None):
        """n (output rows of the largest layer that will be passed): if given, the second context gets a workspace of
        the size slim_workspace_query states for the bit allocation of such a layer, allocated here once, so that no
        call on it allocates; without it the context grows its own.  second = (stream, context): a second stream and
        a context bound to it that the caller keeps (drivers for several shapes share one pair: every new stream may
        land on another hardware queue, and two chains that are meant to overlap can then share one)."""
        self.slim, self.m, self.beta, self.N, self.percdamp, self.t_sba = slim, m, beta, N, percdamp, t_sba
        self.bit_base = binding.bit_base_for(N)     # of the stored form: what its 2-bit group value 0 stands for
        self.G = torch.zeros((m, m), dtype=torch.float32, device=device)
        self.U = torch.empty((m, m), dtype=torch.float64, device=device)
        self.d = torch.empty(m, dtype=torch.float64, device=device)
        self.main = torch.cuda.current_stream()
        self.own_second = second is None
        if second is None:
            self.side = torch.cuda.Stream()
            with torch.cuda.stream(self.side):
                self.slim_sba = binding.Slim(device, 0 if n is None else binding.workspace_query(n, m, beta, 0, t_sba))
        else:
            self.side, self.slim_sba = second

    def contexts(self):
        return [self.slim, self.slim_sba]

    def close(self):
        if self.own_second:
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


def next_layer_input(slim, r, beta, X, n):
    """Calibration activations of the next layer of a chain (Sec. 3.4: every layer inside the GPTQ backbone sees what
    its quantised predecessors emit): the layer of result `r`, applied FROM ITS STORED FORM to the columns of X
    (m x t, fp16, tokens contiguous) by the library's linear-layer kernel (which takes its tokens 16 at a time), rounded to fp16 and
    laid out channels x tokens again.  Only layout changes and the rounding happen here."""
    t = X.shape[1]
    Xn = torch.empty((n, t), dtype=torch.float16, device=X.device)
    step = 4096                                      # tokens per call: bounds the size of the transposed copies
    for t0 in range(0, t, step):
        xin = X[:, t0:t0 + step].t().contiguous()
        y = slim.dequant_matmul(r["packed"], r["gbits"], r["row_off"], r["scale"], r["zero"], beta, xin,
                                bit_base=r["bit_base"])
        Xn[:, t0:t0 + xin.shape[0]] = y.clamp(-65504.0, 65504.0).to(torch.float16).t()
    return Xn


def run_sequential(slim, Ws, X0, beta, N, percdamp=0.01, t_sba=2048):
    """A chain of linear layers quantised in order, each calibrated on the output of its already quantised
    predecessors for the same tokens (the GPTQ backbone that Sec. 3.4 puts SBA and SQC into).  Ws[l] is n_l x m_l
    with m_{l+1} = n_l; X0 is m_0 x t.  Returns the per-layer results of LayerPass.run, each with its calibration
    input under "X" and its packed zero points under "zpacked" (App. B.2)."""
    X, outs = X0, []
    for W in Ws:
        n, m = W.shape
        drv = LayerPass(slim, m, beta, N, percdamp, t_sba, device=str(W.device))
        try:
            r = drv.run(W, X)
        finally:
            drv.close()
        r["X"] = X
        r["zpacked"], _ = slim.pack_zeros(r["zero"], binding.zero_bits_for(N), host_outputs=False)
        outs.append(r)
        X = next_layer_input(slim, r, beta, X, n)
    return outs


def run_plus(slim, W, X, beta, N, steps=20, lr=1e-2, percdamp=0.01, t_sba=2048):
    """SliM-LLM+ on one layer (Sec. 3.4: the bit allocation of SBA plugged into a quantiser with learnable weight
    clipping, trained with AdamW; no SQC, no error compensation): Hessian, inverse, salience and SBA as in the
    plain pass, then slim_lwc_quantize with those widths, then packing of codes and zero points."""
    n, m = W.shape
    G = torch.zeros((m, m), dtype=torch.float32, device=W.device)
    nt = slim.hessian_accumulate(X, G, 0)
    U, d = slim.hessian_inverse(G, nt, percdamp)
    _, grp, _ = slim.salience(W, d, beta)
    bits, _, _ = slim.sba_allocate(W, grp, beta, N, X[:, : min(t_sba, X.shape[1])], host_outputs=False)
    out = slim.lwc_quantize(W, G, nt, bits, beta, steps=steps, lr=lr, host_outputs=False)
    bit_base = binding.bit_base_for(N)
    packed, gbits, row_off, _ = slim.pack(out["codes"], bits, beta, packed_rows=m * (N + 1) // 32, host_outputs=False,
                                          bit_base=bit_base)
    zp, _ = slim.pack_zeros(out["zero"], binding.zero_bits_for(N), host_outputs=False)
    out.update(bits=bits, G=G, n_tokens=nt, bit_base=bit_base, packed=packed, gbits=gbits, row_off=row_off, zpacked=zp,
               m_star=row_off[-1])
    return out
