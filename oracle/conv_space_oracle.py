"""Oracle for the search space of the tunable 2D convolution.  TEST INFRASTRUCTURE ONLY; shares
no code with the library.

Parameters and value lists are those of the paper's table "Best-found parameters for 2D
convolution" and its section "Tuning parameters" (convolution case study):
    Xwg, Ywg in {8,16,32,64}; Xwpt, Ywpt in {1,2,4,8}; L$ in {0,1,2}; VW in {1,2,4,8};
    PAD in {0,1}; UNR in {0,1}.
The constraints are the ones the text states, plus this device's limits:
  * vector operations combine values of one thread, so VW divides Xwpt;
  * PAD pads the local memory, so it is 0 when L$ = 0;
  * a workgroup has at most 1024 threads -- Xwg * Ywg of them, or with L$ = 2
    (Xwg + ceil((Xf-1)/Xwpt)) * (Ywg + ceil((Yf-1)/Ywpt)) including the helper threads;
  * the cached tile fits the 160 KiB of local memory: with L$ = 1 it is
    (Xwg*Xwpt + Xf-1 + PAD) x (Ywg*Ywpt + Yf-1) floats, with L$ = 2 every thread, helpers
    included, caches its Xwpt x Ywpt block, so it is
    ((Xwg + ceil((Xf-1)/Xwpt)) * Xwpt + PAD) x ((Ywg + ceil((Yf-1)/Ywpt)) * Ywpt) floats.

parity unpinned: the paper's count of 3424 valid configurations cannot be reproduced, because
its constraints and device limits are not printed; the counts here are pinned by the counting
argument in the tests (closed form for L$ = 0) and by brute force.
"""
import itertools

NAMES = ("XWG", "YWG", "XWPT", "YWPT", "LMEM", "VW", "PAD", "UNR")
VALUES = ([8, 16, 32, 64], [8, 16, 32, 64], [1, 2, 4, 8], [1, 2, 4, 8], [0, 1, 2], [1, 2, 4, 8],
          [0, 1], [0, 1])
MAX_THREADS = 1024
LDS_LIMIT = 160 * 1024


def _ceil_div(a, b):
    return -(-a // b)


def threads(cfg, Xf, Yf):
    xwg, ywg, xwpt, ywpt, lmem = cfg[:5]
    if lmem == 2:
        return (xwg + _ceil_div(Xf - 1, xwpt)) * (ywg + _ceil_div(Yf - 1, ywpt))
    return xwg * ywg


def lds_bytes(cfg, Xf, Yf):
    xwg, ywg, xwpt, ywpt, lmem, _vw, pad, _unr = cfg
    if lmem == 0:
        return 0
    if lmem == 1:
        return 4 * (xwg * xwpt + Xf - 1 + pad) * (ywg * ywpt + Yf - 1)
    return 4 * ((xwg + _ceil_div(Xf - 1, xwpt)) * xwpt + pad) * \
        ((ywg + _ceil_div(Yf - 1, ywpt)) * ywpt)


def valid(cfg, Xf, Yf):
    xwg, ywg, xwpt, ywpt, lmem, vw, pad, unr = cfg
    if xwpt % vw:
        return False
    if lmem == 0 and pad:
        return False
    if threads(cfg, Xf, Yf) > MAX_THREADS:
        return False
    if lds_bytes(cfg, Xf, Yf) > LDS_LIMIT:
        return False
    return True


def enumerate_space(Xf, Yf):
    """Valid configurations in lexicographic order, first parameter slowest."""
    return [c for c in itertools.product(*VALUES) if valid(c, Xf, Yf)]
