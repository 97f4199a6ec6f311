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


def pack_planes_v2(codes: np.ndarray):
    """FP6 codes uint8 [N,K] -> (hi bytes, lo bytes) in plane layout 2, from the header's description:
    per lane and 32-wide k block, the 192-bit string STR of the 32 codes, split by kind of bit."""
    N, K = codes.shape
    assert N % 64 == 0 and K % 64 == 0
    F = 0xFFFFFFFF
    SE = [sum(1 << p for p in range(32) if (32 * j + p) % 6 >= 2) for j in range(6)]
    MA = [F ^ m for m in SE]
    hi = np.zeros(N * K // 2 // 4, np.uint32)
    lo = np.zeros(N * K // 4 // 4, np.uint32)
    c = codes.reshape(N // 64, 4, 16, K // 64, 2, 4, 8).astype(np.uint64)    # nb, t, n%16, kb, q, k-group, e
    for nb in range(N // 64):
        for kb in range(K // 64):
            ti = nb * (K // 64) + kb
            for q in range(2):
                for lane in range(64):
                    i16, g = lane % 16, lane // 16
                    big = 0
                    for t in range(4):
                        for e in range(8):
                            big |= int(c[nb, t, i16, kb, q, g, e]) << (6 * (8 * t + e))
                    S = [(big >> (32 * j)) & F for j in range(6)]
                    B0 = (S[0] & MA[0]) | (S[1] & MA[1]) | (S[2] & MA[2])
                    B1 = (S[3] & MA[3]) | (S[4] & MA[4]) | (S[5] & MA[5])
                    A0 = (S[0] & SE[0]) | (S[4] & MA[0])
                    A1 = (S[1] & SE[1]) | (((S[4] & 0x0C30C30C) << 2) & F)
                    A2 = (S[2] & SE[2]) | (((S[5] & 0x030C30C3) << 2) & F)
                    r5 = S[5] & 0xF0C30C30
                    A3 = (S[3] & SE[0]) | ((r5 << 2) & F) | (r5 >> 30)
                    lo[(ti * 1024 + lane * 16 + 8 * q) // 4:][:2] = [B0, B1]
                    hi[(ti * 2048 + q * 1024 + lane * 16) // 4:][:4] = [A0, A1, A2, A3]
    return hi.view(np.uint8), lo.view(np.uint8)
