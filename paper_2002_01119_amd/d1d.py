"""Delay-by-one schedule (Sec. 4, D1D-PSGD; Eq. 13 and 14): host-side ordering of the library's kernels.

In D1D-PSGD the gradient used by step k was computed from the previous iterate, Phi_k = W_{k-1}, so the
gradient computation of the NEXT step and the averaging of THIS step are independent and the paper runs
them side by side.  Here the averaging is `psgd.mix_step` / `psgd.mix_full` on one stream and the gradient
producer (the synthetic stand-in `psgd.synth_grad`: G = c * X_prev + noise) runs on a second stream; events
carry the three dependencies that exist:

    mix k          needs  G_k                       (produced on the other stream)
    producer k+1   needs  X_k, which mix k-1 wrote, and the gradient buffer mix k-1 read (two buffers)
    mix k+1        writes the buffer of X_{k-1}, which producer k read: implied, because mix k+1 waits for
                   producer k+1, which follows producer k on its stream

Three X buffers rotate (X_{k-1}, X_k, X_{k+1}); X_k is read by mix k and by producer k+1 at the same time
and written by neither, which is why delay_mode 1 forbids mixing in place.  X_{-1} := X_0.

Only enqueue order lives here: every arithmetic step is a kernel of the library.
"""
import torch

from . import psgd


class DelayByOne:
    """State of a delayed run: the three rotating X buffers, two gradient buffers, streams and events.

    X holds X_0 on entry; Y and X_prev are scratch of the same shape (X_prev is overwritten with X_0).
    `noise` is an [n, d] tensor (used every step) or a callable k -> tensor.  `table` is a callable
    k -> (nbr_dev, w_dev), or None for global averaging (psgd.mix_full).  With overlap=False everything is
    enqueued on `mix_stream` in the serial order producer k, mix k.
    """

    def __init__(self, X, Y, X_prev, Gs, noise, table, lr, c, *, overlap=True, mix_stream=None,
                 producer_stream=None, producer_repeat=1):
        if len(Gs) != 2:
            raise ValueError("two gradient buffers are needed")
        self.X, self.Y, self.X_prev, self.Gs = X, Y, X_prev, list(Gs)
        self.noise = noise if callable(noise) else (lambda k: noise)
        self.table, self.lr, self.c = table, lr, c
        self.overlap = overlap
        self.mix_stream = mix_stream or torch.cuda.current_stream()
        self.producer_stream = producer_stream or (torch.cuda.Stream(device=X.device) if overlap else None)
        self.producer_repeat = max(int(producer_repeat), 1)   # > 1 rewrites the same G again: a slower producer
        self.k = 0
        self._mix_done = {}          # step -> event recorded behind mix k
        self._produced = {}          # step -> event recorded behind the producer of G_k
        with torch.cuda.stream(self.mix_stream):
            self.X_prev.copy_(self.X)                         # X_{-1} := X_0
        if overlap:
            start = torch.cuda.Event()
            start.record(self.mix_stream)
            self.producer_stream.wait_event(start)
            self._produce(0, self.X_prev)

    def _produce(self, k, x_prev):
        s = self.producer_stream if self.overlap else self.mix_stream
        for _ in range(self.producer_repeat):
            psgd.synth_grad(x_prev, self.noise(k), self.Gs[k % 2], self.c, stream=s)
        if self.overlap:
            ev = torch.cuda.Event()
            ev.record(s)
            self._produced[k] = ev

    def step(self, cdist_out=None, before_mix=None, after_mix=None, more=True):
        """Enqueue step k: X_{k+1} = mix(X_k) - lr * G_k with G_k = c * X_{k-1} + noise_k.  `before_mix` /
        `after_mix` are called with the mix stream right around the mix call (for timing events).  `more`
        = False says no further step follows, so no further gradient is produced.  Returns the tensor
        that holds X_{k+1}."""
        k, ms = self.k, self.mix_stream
        G = self.Gs[k % 2]
        if self.overlap:
            ms.wait_event(self._produced.pop(k))
        else:
            self._produce(k, self.X_prev)
        if before_mix:
            before_mix(ms)
        if self.table is None:
            psgd.mix_full(self.X, self.Y, G, self.lr, delay_mode=1, stream=ms, cdist_out=cdist_out)
        else:
            nbr, w = self.table(k)
            psgd.mix_step(self.X, self.Y, G, nbr, w, self.lr, delay_mode=1, stream=ms, cdist_out=cdist_out)
        if after_mix:
            after_mix(ms)
        if self.overlap:
            ev = torch.cuda.Event()
            ev.record(ms)
            self._mix_done[k] = ev
            if more:
                # G_{k+1} = c * X_k + noise: X_k is complete since mix k-1, whose gradient buffer is the one
                # written now; it runs beside mix k, which only reads X_k
                prev = self._mix_done.pop(k - 1, None)
                if prev is not None:
                    self.producer_stream.wait_event(prev)
                self._produce(k + 1, self.X)
        self.X_prev, self.X, self.Y = self.X, self.Y, self.X_prev
        self.k += 1
        return self.X

    def finish(self):
        """Make the mix stream wait for everything enqueued on the producer stream."""
        if self.overlap:
            ev = torch.cuda.Event()
            ev.record(self.producer_stream)
            self.mix_stream.wait_event(ev)
