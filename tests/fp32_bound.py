"""A per-entry bound on how far an fp32-per-operation run of Algorithm 1 (Eq. 7-8) may drift from a run in
double arithmetic that keeps its state in fp32: the tolerance of the fp32-against-double comparisons, derived
instead of observed.

Model: every fp32 operation returns its exact result times (1 + d), |d| <= u = 2^-24 (round to nearest, no
underflow: the tests' magnitudes are far from the denormals).  The errors of the state entering an iteration
(E_w, E_mu, E_v, zero at the start) are pushed through the operations of the iteration in the order of Algorithm 1,
each operation adding u times the magnitude of its result; the double run rounds its state to fp32 when it is
stored, which adds u times the stored value once more.  The scalars 1-beta, 1-alpha, alpha*lambda are formed in
fp32 on one side and in double on the other: relative u each.  Products of two errors are kept where one of the
factors need not be small (the square of the decayed momentum), dropped elsewhere; the final factor 1 + 2^-10
absorbs them.

Three places need more than first order:
* Sign(w) in the decay term: if |w| <= E_w the two runs may see different signs, the term then differs by up to
  2*alpha*lambda;
* the square root: its error is taken from the interval [v^ - E, v^ + E], not from the derivative, because v^ may be
  smaller than its own error;
* the quotient q = mu^/(sqrt(v^) + eps): when the decayed momentum (1-alpha)*mu + alpha*lambda*Sign(w) cancels to
  rounding noise while v is still small, q is noise over noise.  But v_t >= (1-beta2)*mu~^2 in either run, so
  |q| <= sqrt(bc2/(1-beta2))/bc1 in both and they differ by at most twice that: the cap on E_q.  (At the first
  iteration bc2 = 1-beta2 and the cap is 2/bc1 = 20 steps of size lr: the "few lr" such entries are seen to move.)
"""
import numpy as np

U = 2.0 ** -24
SLACK = 1.0 + 2.0 ** -10


class Fp32Drift:
    """Bounds E_w, E_mu, E_v (arrays like the state) after each call of advance()."""

    def __init__(self, shape):
        self.E_w = np.zeros(shape)
        self.E_mu = np.zeros(shape)
        self.E_v = np.zeros(shape)

    def advance(self, w, mu, v, g, keep, *, lr, beta1, beta2, eps, lambda_, alpha, bias_corr1, bias_corr2):
        """w, mu, v: the state of the DOUBLE run entering the iteration (fp32 arrays), g the gradient both runs
        receive, keep the mask (0/1) both runs apply; the scalars as the fp32 values both runs are given."""
        f = lambda x: float(np.float32(x))
        lr, b1, b2, eps, lam, al_, bc1, bc2 = map(f, (lr, beta1, beta2, eps, lambda_, alpha, bias_corr1, bias_corr2))
        w, mu, v, g = (np.asarray(x, np.float64) for x in (w, mu, v, g))
        kept = np.asarray(keep).astype(bool)
        c1, c2, oma, al = 1.0 - b1, 1.0 - b2, 1.0 - al_, al_ * lam
        # first moment
        t0, t1 = b1 * mu, c1 * g
        mu_t = t0 + t1
        E_t0 = b1 * self.E_mu + U * np.abs(t0)
        E_t1 = 2 * U * np.abs(t1)
        E_mut = E_t0 + E_t1 + U * np.abs(mu_t)
        # decayed momentum on the entries that are not kept (Eq. 7)
        d0, d1 = oma * mu_t, al * np.sign(w)
        dec = d0 + d1
        E_d0 = oma * E_mut + 2 * U * np.abs(d0)
        E_d1 = U * np.abs(d1) + np.where(np.abs(w) <= self.E_w, 2 * abs(al), 0.0)
        E_dec = E_d0 + E_d1 + U * np.abs(dec)
        mt = np.where(kept, mu_t, dec)
        E_mt = np.where(kept, E_mut, E_dec)
        # second moment from the decayed momentum (Eq. 8)
        sq = mt * mt
        E_sq = 2 * np.abs(mt) * E_mt + E_mt ** 2 + U * sq
        s0, s1 = b2 * v, c2 * sq
        E_s0 = b2 * self.E_v + U * s0
        E_s1 = c2 * E_sq + 2 * U * s1
        v_t = s0 + s1
        E_vt = E_s0 + E_s1 + U * v_t
        # bias corrections, square root, quotient
        mh, vh = mt / bc1, v_t / bc2
        E_mh = E_mt / bc1 + U * np.abs(mh)
        E_vh = E_vt / bc2 + U * vh
        r = np.sqrt(vh)
        E_r = np.maximum(np.sqrt(vh + E_vh) - r, r - np.sqrt(np.maximum(vh - E_vh, 0.0))) + U * r
        den = r + eps
        E_den = E_r + U * den
        den_lo = np.maximum(den - E_den, eps * (1 - 2 * U))
        q_mag = (np.abs(mh) + E_mh) / den_lo
        E_q = E_mh / den_lo + np.abs(mh) * E_den / (den * den_lo) + U * q_mag
        q_cap = np.sqrt(bc2 / c2) / bc1 * (1 + 16 * U)      # |q| in either run
        E_q = np.minimum(E_q, 2 * q_cap)
        step_mag = lr * np.minimum(q_mag, q_cap)
        E_step = lr * E_q + U * step_mag
        w_new = w - lr * (mh / den)
        # what is stored: mu (not mu~), v, w; the double run rounds each to fp32 on store
        self.E_mu = (E_mut + U * np.abs(mu_t)) * SLACK
        self.E_v = (E_vt + U * v_t) * SLACK
        self.E_w = (self.E_w + E_step + 2 * U * (np.abs(w_new) + self.E_w + E_step)) * SLACK

    def scalars(self, cfg):
        """The keyword arguments of advance() from an object with the oracle's configuration fields."""
        return dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, lambda_=cfg.lambda_, alpha=cfg.alpha,
                    bias_corr1=cfg.bias_corr1, bias_corr2=cfg.bias_corr2)
