"""CPU oracle of the progressive-resolution stage switch (Sec. 3.2, Eq. 4).  TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; the
product path (paper_2505_16864_amd) never does.  Plain float64 numpy, loops over output cells,
no blocking or fusion.

Eq. 4:   x_{t-1} = (1 - sigma_t) * U(x0_hat) + sigma_t * eps_tilde,   x0_hat = x_t - sigma_t * eps_t

U is "area interpolation" in 3D.  The paper does not define it further; the reading taken here is
the one the name has in deep-learning libraries (adaptive average pooling): along each axis with I
input and O output cells, output cell o is the unweighted mean of input cells
floor(o*I/O) .. ceil((o+1)*I/O) - 1, and the 3D operator is the product of the three 1D ones.
The Gaussian draw eps_tilde is an input (the caller owns the random stream).
"""
import numpy as np


def area_window(o, n_in, n_out):
    """[start, end) of the input cells that output cell o averages (Sec. 3.2, U of Eq. 4)."""
    start = (o * n_in) // n_out
    end = -((-(o + 1) * n_in) // n_out)          # ceil((o+1)*n_in/n_out) in integers
    return start, end


def upsample_area(x, out_shape):
    """U(x): x is [C, T, H, W] float64; out_shape = (T', H', W')."""
    x = np.asarray(x, dtype=np.float64)
    C, T, H, W = x.shape
    To, Ho, Wo = out_shape
    out = np.empty((C, To, Ho, Wo), dtype=np.float64)
    for t in range(To):
        t0, t1 = area_window(t, T, To)
        for h in range(Ho):
            h0, h1 = area_window(h, H, Ho)
            for w in range(Wo):
                w0, w1 = area_window(w, W, Wo)
                out[:, t, h, w] = x[:, t0:t1, h0:h1, w0:w1].mean(axis=(1, 2, 3))
    return out


def stage_switch(x_t, eps_t, eps_tilde, sigma_t, out_shape):
    """Eq. 4.  x_t, eps_t: [C, T, H, W]; eps_tilde: [C, T', H', W']; returns x_{t-1} [C, T', H', W']."""
    x_t = np.asarray(x_t, dtype=np.float64)
    x0_hat = x_t - sigma_t * np.asarray(eps_t, dtype=np.float64)
    return (1.0 - sigma_t) * upsample_area(x0_hat, out_shape) + sigma_t * np.asarray(eps_tilde, dtype=np.float64)
