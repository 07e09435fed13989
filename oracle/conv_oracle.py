"""Oracle for the 2D convolution of the paper's first case study.  TEST INFRASTRUCTURE ONLY;
shares no code with the library.

The section "Case-study: 2D convolution" defines, for an Xf x Yf filter F, an input image A and
a weighing factor w,

    B[x, y] = w * sum_{i} sum_{j} F[i, j] * A[x + i, y + j]

with i and j running over the filter, centred on (x, y); the output image has X x Y points.
Readings taken here (the paper does not say what happens at the image border): the input is
stored WITH its halo, (Y + Yf - 1) rows of (X + Xf - 1) values, so that every tap of every output
exists, and indices are shifted to start at zero -- output row y, column x reads input rows
y .. y + Yf - 1 and columns x .. x + Xf - 1.  Arrays are row-major with x the fastest index.
The filter is NOT flipped (the formula adds F[i, j] * A[x + i, y + j]: a correlation).

`conv2d(...)` writes that definition out with numpy in float64 (one shifted slice of the image
per filter tap); `conv2d_python(...)` is the same sum as plain Python loops, for tiny inputs;
`tolerance(...)` is the per-element bound a float32 implementation must meet:
    |B_gpu - B_ref| <= 1e-5 * Xf * Yf * |w| * max|F| * max|A| + 1e-6 * |B_ref|
(the GEMM bound of this build with the Xf*Yf taps of one output in the place of K).
"""
import numpy as np


def conv2d(A, F, w, X, Y):
    """A: (Y + Yf - 1, >= X + Xf - 1) float array, F: (Yf, Xf).  Returns (Y, X) float64."""
    A = np.asarray(A, dtype=np.float64)
    F = np.asarray(F, dtype=np.float64)
    Yf, Xf = F.shape
    if A.shape[0] < Y + Yf - 1 or A.shape[1] < X + Xf - 1:
        raise ValueError("the input image must hold the halo: (Y+Yf-1) x (X+Xf-1)")
    B = np.zeros((Y, X), dtype=np.float64)
    for j in range(Yf):
        for i in range(Xf):
            B += F[j, i] * A[j:j + Y, i:i + X]
    return float(w) * B


def conv2d_python(A, F, w, X, Y):
    Yf, Xf = len(F), len(F[0])
    B = [[0.0] * X for _ in range(Y)]
    for y in range(Y):
        for x in range(X):
            s = 0.0
            for j in range(Yf):
                for i in range(Xf):
                    s += float(F[j][i]) * float(A[y + j][x + i])
            B[y][x] = float(w) * s
    return B


def conv2d_sample(A, F, w, ys, xs):
    """The same values for chosen outputs (ys[n], xs[n]) only: for full-size images."""
    A = np.asarray(A)
    F = np.asarray(F, dtype=np.float64)
    Yf, Xf = F.shape
    out = np.empty(len(ys), dtype=np.float64)
    for n, (y, x) in enumerate(zip(ys, xs)):
        out[n] = float(w) * np.sum(F * A[y:y + Yf, x:x + Xf].astype(np.float64))
    return out


def tolerance(B_ref, F, A_used, w):
    F = np.asarray(F)
    amax = float(np.max(np.abs(A_used))) if np.size(A_used) else 0.0
    fmax = float(np.max(np.abs(F))) if F.size else 0.0
    return 1e-5 * F.size * abs(float(w)) * fmax * amax + 1e-6 * np.abs(B_ref)
