"""Partial gradients g_j = sum over the rows of block j of grad_theta L  (Sec. II-C).

The sum is NOT divided by the number of rows: the update rule (Sec. II-B,
eq. (1)) applies eta/m to the summed gradient.  The paper leaves the loss
generic; the three below are the textbook ones used by the workloads.  All
arithmetic in fp64.  TEST INFRASTRUCTURE ONLY.
"""
import numpy as np


def _f64(a):
    return np.asarray(a, dtype=np.float64)


def lsq_loss(X, y, theta):
    """L = 1/2 sum_i (x_i.theta - y_i)^2."""
    r = _f64(X) @ _f64(theta) - _f64(y)
    return 0.5 * float(r @ r)


def lsq_gradient(X, y, theta):
    """g = X^T (X theta - y) for one row block."""
    X = _f64(X)
    return X.T @ (X @ _f64(theta) - _f64(y))


def logistic_loss(X, y, theta):
    """L = sum_i log(1 + exp(-y_i x_i.theta)), labels y_i in {-1,+1}."""
    z = _f64(y) * (_f64(X) @ _f64(theta))
    return float(np.sum(np.logaddexp(0.0, -z)))


def logistic_gradient(X, y, theta):
    """g = - sum_i y_i x_i / (1 + exp(y_i x_i.theta))."""
    X = _f64(X)
    y = _f64(y)
    z = y * (X @ _f64(theta))
    # 1/(1+e^z) written so that neither branch overflows
    sig = np.where(z >= 0, np.exp(-np.abs(z)) / (1.0 + np.exp(-np.abs(z))),
                   1.0 / (1.0 + np.exp(-np.abs(z))))
    return X.T @ (-y * sig)


def mlp2_unpack(theta, d_in, hidden, classes):
    """theta = [W1 (d_in x hidden) | b1 (hidden) | W2 (hidden x classes) | b2 (classes)]."""
    theta = _f64(theta)
    o = 0
    W1 = theta[o:o + d_in * hidden].reshape(d_in, hidden); o += d_in * hidden
    b1 = theta[o:o + hidden]; o += hidden
    W2 = theta[o:o + hidden * classes].reshape(hidden, classes); o += hidden * classes
    b2 = theta[o:o + classes]; o += classes
    assert o == theta.size
    return W1, b1, W2, b2


def mlp2_loss(X, labels, theta, hidden, classes):
    """Softmax cross-entropy of a 2-layer ReLU network, summed over rows."""
    X = _f64(X)
    W1, b1, W2, b2 = mlp2_unpack(theta, X.shape[1], hidden, classes)
    H = np.maximum(X @ W1 + b1, 0.0)
    Z2 = H @ W2 + b2
    Z2 = Z2 - Z2.max(axis=1, keepdims=True)
    logp = Z2 - np.log(np.exp(Z2).sum(axis=1, keepdims=True))
    return float(-logp[np.arange(X.shape[0]), np.asarray(labels)].sum())


def mlp2_gradient(X, labels, theta, hidden, classes):
    """Back-propagated gradient of mlp2_loss, in the layout of theta.

    ReLU'(0) is taken as 0; softmax subtracts the row maximum first.
    """
    X = _f64(X)
    labels = np.asarray(labels)
    W1, b1, W2, b2 = mlp2_unpack(theta, X.shape[1], hidden, classes)
    Z1 = X @ W1 + b1
    H = np.maximum(Z1, 0.0)
    Z2 = H @ W2 + b2
    E = np.exp(Z2 - Z2.max(axis=1, keepdims=True))
    P = E / E.sum(axis=1, keepdims=True)
    dZ2 = P
    dZ2[np.arange(X.shape[0]), labels] -= 1.0
    dW2 = H.T @ dZ2
    db2 = dZ2.sum(axis=0)
    dZ1 = (dZ2 @ W2.T) * (Z1 > 0.0)
    dW1 = X.T @ dZ1
    db1 = dZ1.sum(axis=0)
    return np.concatenate([dW1.ravel(), db1, dW2.ravel(), db2])


def partial_gradients(loss, X, Y, theta, hidden=0, classes=0):
    """G = (g_1 ... g_k)^T for X [k, rows, d_in], Y [k, rows]  (Sec. II-C)."""
    rows = []
    for j in range(len(X)):
        if loss == 0:
            rows.append(lsq_gradient(X[j], Y[j], theta))
        elif loss == 1:
            rows.append(logistic_gradient(X[j], Y[j], theta))
        elif loss == 2:
            rows.append(mlp2_gradient(X[j], Y[j], theta, hidden, classes))
        else:
            raise ValueError("unknown loss %r" % (loss,))
    return np.stack(rows)


def gd_update(theta, g, eta, m):
    """theta <- theta - (eta/m) g   (Sec. II-B, eq. (1))."""
    return _f64(theta) - (eta / m) * _f64(g)
