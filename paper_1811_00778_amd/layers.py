"""Index tables that express network layers as gather rows for hcnn_ct_scalar_mac.

One ciphertext per neuron (Sec. 3.1, pixel-per-ciphertext packing): a feature map
[C][H][W] is the ciphertext list with index c*H*W + r*W + x.  Pure indexing, no
arithmetic of the scheme.
"""
import numpy as np


def conv_index_table(c_in, h, w, fh, fw, stride, pad=0):
    """Gather rows of a convolution without bias.

    Returns (idx [G][T] uint32, valid [G][T] bool, (h_out, w_out)); G = h_out*w_out placements in
    row-major order, T = c_in*fh*fw terms in (channel, dy, dx) order.  The top-left input of
    placement (j, kk) is j*stride*w + kk*stride, the rule f_jk = j*s_h*i_w + k*s_w of Sec. 4.4.1.
    With pad > 0, terms that fall outside the image have valid = False (their index is 0 and the
    caller must give them weight 0).
    """
    h_out = (h + 2 * pad - fh) // stride + 1
    w_out = (w + 2 * pad - fw) // stride + 1
    G, T = h_out * w_out, c_in * fh * fw
    idx = np.zeros((G, T), dtype=np.uint32)
    valid = np.ones((G, T), dtype=bool)
    for j in range(h_out):
        for kk in range(w_out):
            g = j * w_out + kk
            tau = 0
            for c in range(c_in):
                for dy in range(fh):
                    for dx in range(fw):
                        r, x = j * stride + dy - pad, kk * stride + dx - pad
                        if 0 <= r < h and 0 <= x < w:
                            idx[g, tau] = c * h * w + r * w + x
                        else:
                            valid[g, tau] = False
                        tau += 1
    return idx, valid, (h_out, w_out)


def conv_weight_table(weights, n_groups, valid=None):
    """weights [F][c_in][fh][fw] -> w [G][F][T] int32 (the same filter bank at every placement)."""
    F = weights.shape[0]
    flat = np.ascontiguousarray(weights.reshape(F, -1), dtype=np.int32)
    w = np.broadcast_to(flat[None, :, :], (n_groups,) + flat.shape).copy()
    if valid is not None:
        w *= valid[:, None, :].astype(np.int32)
    return w


def pool_index_table(channels, h, w, extent, stride=None):
    """Average pooling as the paper evaluates it (Sec. 4.3): a convolution with all-ones weights per
    channel (the division by the window size is folded into the layer's scale factor).

    Returns (idx [G][T] uint32, ones [G][1][T] int32, (h_out, w_out)); G = channels*h_out*w_out groups in
    (channel, row, column) order -- which is the output feature-map order -- and T = extent*extent."""
    stride = extent if stride is None else stride
    h_out, w_out = (h - extent) // stride + 1, (w - extent) // stride + 1
    G, T = channels * h_out * w_out, extent * extent
    idx = np.zeros((G, T), dtype=np.uint32)
    g = 0
    for c in range(channels):
        for j in range(h_out):
            for kk in range(w_out):
                tau = 0
                for dy in range(extent):
                    for dx in range(extent):
                        idx[g, tau] = c * h * w + (j * stride + dy) * w + (kk * stride + dx)
                        tau += 1
                g += 1
    return idx, np.ones((G, 1, T), dtype=np.int32), (h_out, w_out)


def fc_index_table(n_in):
    """Fully connected layer: one group whose gather row lists every input."""
    return np.arange(n_in, dtype=np.uint32)[None, :]


def fc_weight_table(weights):
    """weights [n_out][n_in] -> w [1][n_out][n_in] int32."""
    return np.ascontiguousarray(weights, dtype=np.int32)[None, :, :]
