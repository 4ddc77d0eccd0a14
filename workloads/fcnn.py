"""A quantised fully connected ReLU network, run forward and backward in exact
integers, to produce the tensors of one aggregation window.

Fixed point: scale 2^16 (R = 16), activations / weights / gradients held as
32-bit integers, pre-activations Z and activation gradients G_A at scale 2^32
as 48-bit integers (Q = 32).  Rescaling is round-half-up,
(x + 2^(R-1)) >> R with an arithmetic shift, followed by ReLU gated on Z >= 0.
Matrix products run in float64 BLAS; every partial sum is an integer below 2^53
in magnitude (asserted from the operands' maxima), so they are exact.
"""
import numpy as np

SCALE_BITS = 16


def quantise(x, bits=SCALE_BITS):
    """floor(x * 2^bits + 1/2) as int64; asserted to fit int32."""
    q = np.floor(np.asarray(x, dtype=np.float64) * float(1 << bits) + 0.5).astype(np.int64)
    assert q.min(initial=0) >= -(1 << 31) and q.max(initial=0) < (1 << 31)
    return q


def _exact_matmul(a, b):
    a = np.asarray(a, dtype=np.int64)
    b = np.asarray(b, dtype=np.int64)
    bound = int(np.abs(a).max(initial=0)) * int(np.abs(b).max(initial=0)) * a.shape[-1]
    assert bound < (1 << 53), "float64 matmul would not be exact"
    return np.rint(a.astype(np.float64) @ b.astype(np.float64)).astype(np.int64)


def _rescale(x, bits=SCALE_BITS):
    return (x + (1 << (bits - 1))) >> bits


def _rescale_nearest(x, bits):
    """x / 2^bits to the nearest integer, halves away from zero (the rule of the weight update)."""
    mag = (np.abs(x) + (1 << (bits - 1))) >> bits
    return np.where(x >= 0, mag, -mag)


def fc_relu_layer(seed, batch=16, width=256):
    """One FC layer + ReLU: X [batch,width] ~ U[0,1), W [width,width] ~ N(0, 2/width),
    both quantised at 2^16; Z = X W as 48-bit integers."""
    rng = np.random.default_rng(seed)
    x = quantise(rng.random((batch, width)))
    w = quantise(rng.normal(0.0, np.sqrt(2.0 / width), (width, width)))
    z = _exact_matmul(x, w)
    assert np.abs(z).max() < (1 << 47)
    return dict(X=x.astype(np.int32), W=w.astype(np.int32), Z=z)


def fcnn_window(seed, n_layers, width, batch, steps=1, lr_shift=None, q_bits=32, r_bits=SCALE_BITS):
    """T' = `steps` consecutive SGD steps of an L-layer width x width network.

    Step t draws its batch A^(0) ~ U[0,1) and output gradient dL/dY ~ N(0, 1e-2)
    (variance) from default_rng(seed + 1 + t); weights ~ N(0, 2/width) from
    default_rng(seed) before step 0.  Between steps W <- W - G_W / 2^(16 + lr_shift) rounded to nearest
    (halves away from zero);
    by default lr_shift = 8 + log2(batch): learning rate 2^-8 on the batch-mean gradient
    (with the summed gradient the random output gradients make the weights, and then the
    activations, leave the 32-bit range within a few steps).
    Returns stacks with slot n = t L + (l-1):
      A  int32 [N,B,w]  input of layer l (A^(l-1))
      W  int32 [N,w,w]  weights of layer l at step t
      GZ int32 [N,B,w]  gradient of Z^(l)
      Zr int64 [N,B,w]  Z^(l) where a ReLU follows (l < L), else 0
      GA int64 [N,B,w]  gradient of A^(l) before rescaling (l < L), else 0
    """
    if lr_shift is None:
        lr_shift = 8 + int(batch).bit_length() - 1
    wrng = np.random.default_rng(seed)
    weights = [quantise(wrng.normal(0.0, np.sqrt(2.0 / width), (width, width)))
               for _ in range(n_layers)]
    n = n_layers * steps
    a_st = np.zeros((n, batch, width), dtype=np.int32)
    w_st = np.zeros((n, width, width), dtype=np.int32)
    gz_st = np.zeros((n, batch, width), dtype=np.int32)
    zr_st = np.zeros((n, batch, width), dtype=np.int64)
    ga_st = np.zeros((n, batch, width), dtype=np.int64)
    lim_in = 1 << (q_bits + r_bits - 1)
    lim_q = 1 << (q_bits - 1)
    for t in range(steps):
        rng = np.random.default_rng(seed + 1 + t)
        act = quantise(rng.random((batch, width)))
        zs = []
        for l in range(n_layers):
            k = t * n_layers + l
            a_st[k] = act
            w_st[k] = weights[l]
            z = _exact_matmul(act, weights[l])
            zs.append(z)
            if l < n_layers - 1:
                assert np.abs(z).max() < lim_in
                zr_st[k] = z
                zp = _rescale(z)
                assert zp.min() >= -lim_q and zp.max() < lim_q
                act = np.where(z >= 0, zp, 0)
        g_z = quantise(rng.normal(0.0, 0.1, (batch, width)))
        new_weights = list(weights)
        for l in range(n_layers - 1, -1, -1):
            k = t * n_layers + l
            gz_st[k] = g_z
            g_w = _exact_matmul(a_st[k].T, g_z)
            new_weights[l] = weights[l] - _rescale_nearest(g_w, SCALE_BITS + lr_shift)
            assert np.abs(new_weights[l]).max() < (1 << 31)
            if l > 0:
                g_a = _exact_matmul(g_z, weights[l].T)
                assert np.abs(g_a).max() < lim_in
                ga_st[k - 1] = g_a
                gap = _rescale(g_a)
                assert gap.min() >= -lim_q and gap.max() < lim_q
                g_z = np.where(zs[l - 1] >= 0, gap, 0)
        weights = new_weights
    return dict(L=n_layers, B=batch, width=width, T=steps, Q=q_bits, R=r_bits,
                A=a_st, W=w_st, GZ=gz_st, Zr=zr_st, GA=ga_st)
