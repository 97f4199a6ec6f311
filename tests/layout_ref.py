"""numpy statement of the plane layout documented in include/fp6_linear.h (layout
version 1), written from that text only.  It lets the tests turn the oracle's codes
into the exact bytes the library must produce, and build planes for arbitrary codes.
Test infrastructure: neither the oracle nor the library uses it."""
import numpy as np


def pack_planes(codes: np.ndarray):
    """codes uint8 [N,K] (s<<5|eee<<2|mm) -> (hi bytes [N*K/2], lo bytes [N*K/4])."""
    N, K = codes.shape
    assert N % 64 == 0 and K % 64 == 0
    n = np.arange(N)[:, None]
    k = np.arange(K)[None, :]
    nn, kk = n % 64, k % 64
    ti = (n // 64) * (K // 64) + (k // 64)
    lane = 16 * ((kk % 32) // 8) + (nn % 16)
    f = 2 * (nn // 16) + (kk // 32)
    e = kk % 8
    grp, j = e // 4, e % 4
    b = 2 * (j & 1) + (j >> 1)
    c = codes.astype(np.uint32)
    s, ex, m = c >> 5, (c >> 2) & 7, c & 3

    hi_addr = ti * 2048 + (f // 4) * 1024 + lane * 16 + (f % 4) * 4 + b
    hi_val = (s << grp) | (ex << (2 + 3 * grp))
    hi = np.zeros(N * K // 2, np.uint32)
    np.bitwise_or.at(hi, (hi_addr + 0 * c).ravel(), hi_val.ravel())

    lo_addr = ti * 1024 + lane * 16 + (f // 2) * 4 + b
    lo_val = m << (4 * (f % 2) + 2 * grp)
    lo = np.zeros(N * K // 4, np.uint32)
    np.bitwise_or.at(lo, (lo_addr + 0 * c).ravel(), lo_val.ravel())
    return hi.astype(np.uint8), lo.astype(np.uint8)


def pack_planes5(codes: np.ndarray):
    """FP5 codes uint8 [N,K] (s<<4|eee<<1|m) -> (hi bytes [N*K/2], lo bytes [N*K/8]); the 4-bit plane
    is laid out like the FP6 one, the 1-bit plane as the header's FP5 paragraph says."""
    N, K = codes.shape
    assert N % 64 == 0 and K % 64 == 0
    n = np.arange(N)[:, None]
    k = np.arange(K)[None, :]
    nn, kk = n % 64, k % 64
    ti = (n // 64) * (K // 64) + (k // 64)
    lane = 16 * ((kk % 32) // 8) + (nn % 16)
    f = 2 * (nn // 16) + (kk // 32)
    e = kk % 8
    grp, j = e // 4, e % 4
    b = 2 * (j & 1) + (j >> 1)
    c = codes.astype(np.uint32)
    s, ex, m = c >> 4, (c >> 1) & 7, c & 1

    hi_addr = ti * 2048 + (f // 4) * 1024 + lane * 16 + (f % 4) * 4 + b
    hi_val = (s << grp) | (ex << (2 + 3 * grp))
    hi = np.zeros(N * K // 2, np.uint32)
    np.bitwise_or.at(hi, (hi_addr + 0 * c).ravel(), hi_val.ravel())

    lo_addr = ti * 512 + lane * 8 + (f // 4) * 4 + b
    lo_val = m << (2 * (f % 4) + grp)
    lo = np.zeros(N * K // 8, np.uint32)
    np.bitwise_or.at(lo, (lo_addr + 0 * c).ravel(), lo_val.ravel())
    return hi.astype(np.uint8), lo.astype(np.uint8)
