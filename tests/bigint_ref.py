"""A second, even slower definition of the bootstrapping, in Python integers, for tiny parameters.

It is written from the mathematics rather than from the C oracle: polynomial products go through the
explicit N x N negacyclic matrix of one operand, the gadget digits are the unique balanced base-B
representation of the rounded value, rounding is done with exact integer floor divisions.  The C oracle
must agree with it bit for bit (brute force on tiny inputs).
"""
Q = 1 << 64


def negacyclic_matrix(P):
    """M[c][b] such that (P * Q)[c] = sum_b M[c][b] Q[b]  in Z[X]/(X^N+1)."""
    N = len(P)
    M = [[0] * N for _ in range(N)]
    for c in range(N):
        for b in range(N):
            a = c - b
            M[c][b] = P[a] if a >= 0 else -P[a + N]
    return M


def polymul(P, Qp):
    M = negacyclic_matrix(P)
    return [sum(M[c][b] * Qp[b] for b in range(len(P))) % Q for c in range(len(P))]


def monomial(P, r):
    """X^r * P through an explicit polynomial multiplication with the monomial."""
    N = len(P)
    r %= 2 * N
    mono = [0] * N
    if r < N:
        mono[r] = 1
    else:
        mono[r - N] = -1
    return polymul(mono, P)


def round_shift(x, drop_bits):
    """floor(x / 2^drop + 1/2) for a non-negative integer x."""
    if drop_bits == 0:
        return x
    return (x + (1 << (drop_bits - 1))) >> drop_bits


def digits(x, beta, level):
    """Balanced base-2^beta digits (most significant first) of round(x / 2^(64 - beta*level)) mod 2^(beta*level)."""
    B = 1 << beta
    R = round_shift(x % Q, 64 - beta * level) % (1 << (beta * level))
    out = []
    for _ in range(level):
        d = ((R + B // 2) % B) - B // 2      # representative of R mod B in [-B/2, B/2)
        out.append(d)
        R = (R - d) // B
    return out[::-1]                         # the final R (0 or 1) is the dropped carry


def modswitch(x, N):
    return round_shift((x % Q) * 2 * N, 64) % (2 * N)


def blind_rotate(params, lwe, lut, bsk, n_steps):
    n, k, N, beta, level = params
    bt = modswitch(lwe[n], N)
    acc = [[0] * N for _ in range(k)] + [monomial(lut, -bt)]
    for i in range(n_steps):
        at = modswitch(lwe[i], N)
        lam = []
        for r in range(k + 1):
            rot = monomial(acc[r], at)
            lam.append([(rot[c] - acc[r][c]) % Q for c in range(N)])
        new = [list(comp) for comp in acc]
        for r in range(k + 1):
            dig = [digits(v, beta, level) for v in lam[r]]
            for j in range(level):
                dpoly = [dig[c][j] for c in range(N)]
                for comp in range(k + 1):
                    prod = polymul(dpoly, bsk[i][r][j][comp])
                    new[comp] = [(new[comp][c] + prod[c]) % Q for c in range(N)]
        acc = new
    return acc


def sample_extract(params, acc):
    n, k, N, beta, level = params
    out = []
    for r in range(k):
        # coefficient j of the extracted mask pairs with key coefficient j: X^0 coefficient of A_r * S_r
        out += [acc[r][0]] + [(-acc[r][N - j]) % Q for j in range(1, N)]
    return out + [acc[k][0]]


def keyswitch(lwe_big, ksk, beta, level, n):
    out = [0] * n + [lwe_big[-1]]
    for i, a in enumerate(lwe_big[:-1]):
        for j, d in enumerate(digits(a, beta, level)):
            for x in range(n + 1):
                out[x] = (out[x] - d * ksk[i][j][x]) % Q
    return out
