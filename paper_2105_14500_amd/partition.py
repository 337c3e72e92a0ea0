"""Host-side block views of the Tesseract partition (Alg. 3 and Section 3.1).

Pure index arithmetic on tensors that already live on the device: each helper
returns the q panels that processor (i,j,k) would receive over the q steps, as
strided views (no copies) of unpartitioned matrices, plus the place of its
output block.  Used to emulate a whole [q,q,d] grid sequentially on one GPU.
"""


def block_dims(q, d, a, b, c):
    if not (1 <= d <= q):
        raise ValueError("need 1 <= d <= q")
    if a % (q * d) or b % q or c % q:
        raise ValueError("a must divide by q*d, b and c by q")
    return a // (q * d), b // q, c // q


def block_row(q, i, k):
    """Block row of A and C that processor (i, ., k) holds: h = i + k*q."""
    return i + k * q


def fwd_panels(X, W, q, d, i, j, k):
    """Panels of step t: A_{i,t,k} = block (h, t) of X, B_{t,j} = block (t, j) of W."""
    a, b = X.shape
    c = W.shape[1]
    m, kb, n = block_dims(q, d, a, b, c)
    h = block_row(q, i, k)
    a_p = [X[h * m:(h + 1) * m, t * kb:(t + 1) * kb] for t in range(q)]
    b_p = [W[t * kb:(t + 1) * kb, j * n:(j + 1) * n] for t in range(q)]
    return a_p, b_p


def out_block(C, q, d, i, j, k):
    """View of the block of an [a, *]-shaped matrix that processor (i,j,k) owns."""
    a, c = C.shape
    m, n = a // (q * d), c // q
    h = block_row(q, i, k)
    return C[h * m:(h + 1) * m, j * n:(j + 1) * n]


def dx_panels(dY, W, q, d, i, j, k):
    """dX_{i,j,k} needs dY_{i,t,k} = block (h, t) of dY and W_{j,t} = block (j, t) of W."""
    a, c = dY.shape
    b = W.shape[0]
    m, kb, n = block_dims(q, d, a, b, c)
    h = block_row(q, i, k)
    dy_p = [dY[h * m:(h + 1) * m, t * n:(t + 1) * n] for t in range(q)]
    w_p = [W[j * kb:(j + 1) * kb, t * n:(t + 1) * n] for t in range(q)]
    return dy_p, w_p


def dw_panels(X, dY, q, d, i, j, k):
    """dW^(k)_{i,j} needs X_{t,i,k} = block (t + k*q, i) of X and dY_{t,j,k} = block
    (t + k*q, j) of dY."""
    a, b = X.shape
    c = dY.shape[1]
    m, kb, n = block_dims(q, d, a, b, c)
    x_p, dy_p = [], []
    for t in range(q):
        h = block_row(q, t, k)
        x_p.append(X[h * m:(h + 1) * m, i * kb:(i + 1) * kb])
        dy_p.append(dY[h * m:(h + 1) * m, j * n:(j + 1) * n])
    return x_p, dy_p


def weight_block(W, q, i, j):
    """View of block (i, j) of a [b, c] weight-shaped matrix."""
    b, c = W.shape
    kb, n = b // q, c // q
    return W[i * kb:(i + 1) * kb, j * n:(j + 1) * n]
