"""Brute-force big-integer evaluation of the definitions, for tiny inputs only.

Pure Python, arbitrary-precision integers, no shortcuts: a third, independent
evaluation used to pin the C oracle (never the other way round).
Follows the paper's Section 2.2 (shingles, H hashes, minimum), Eq. 1 of
Section 3.2 (polynomial shingle hash) and Section 2.3 (bands).
"""
P = (1 << 61) - 1
Q = 257
QB = 1687994237021934823
GA = 1425089352415399810
GB = 955111447119501601


P_PAPER = 4294967            # Section 3.2: the modulus of the paper's experiments


def eq1(s: bytes, q: int = Q, p: int = P) -> int:
    return sum(c * q ** i for i, c in enumerate(s)) % p


def shingle_strings(text: bytes, n: int, byte_mode: bool):
    if byte_mode:
        if len(text) == 0:
            return []
        if len(text) < n:
            return [text]
        return [text[i:i + n] for i in range(len(text) - n + 1)]
    toks = text.split()          # bytes.split(): ASCII whitespace 09-0D and 20
    if not toks:
        return []
    if len(toks) < n:
        return [b" ".join(toks)]
    return [b" ".join(toks[i:i + n]) for i in range(len(toks) - n + 1)]


def coeffs(seed: int, K: int):
    s0 = seed % (P - 1) + 1
    a = [s0 * pow(GA, k + 1, P) % P for k in range(K)]
    b = [s0 * pow(GB, k + 1, P) % P for k in range(K)]
    return a, b


def signature(text: bytes, n: int, K: int, seed: int = 0, byte_mode: bool = False):
    a, b = coeffs(seed, K)
    xs = [eq1(s) for s in shingle_strings(text, n, byte_mode)]
    return [min(((a[k] * x + b[k]) % P) % (1 << 32) for x in xs) if xs else 0xFFFFFFFF
            for k in range(K)]


def band_keys(sig, b: int, r: int):
    return [sum(sig[j * r + i] * QB ** i for i in range(r)) % P for j in range(b)]


def clusters(keys):
    """keys: list of per-doc lists; O(n^2 b) edges, then label propagation to a fixed point."""
    n = len(keys)
    label = list(range(n))
    changed = True
    while changed:
        changed = False
        for u in range(n):
            for v in range(u + 1, n):
                if any(ku == kv for ku, kv in zip(keys[u], keys[v])):
                    m = min(label[u], label[v])
                    if label[u] != m or label[v] != m:
                        label[u] = label[v] = m
                        changed = True
    return label


def jaccard(text_a: bytes, text_b: bytes, n: int, byte_mode: bool = False) -> float:
    A = set(shingle_strings(text_a, n, byte_mode))
    B = set(shingle_strings(text_b, n, byte_mode))
    if not A and not B:
        return 1.0
    return len(A & B) / len(A | B)


# ---- paper-prime mode: Eq. 1 and the H functions modulo the paper's own p ----

def coeffs_pp(seed: int, K: int):
    a, b = coeffs(seed, K)
    return [x % (P_PAPER - 1) + 1 for x in a], [x % P_PAPER for x in b]


def signature_pp(text: bytes, n: int, K: int, seed: int = 0, byte_mode: bool = False):
    a, b = coeffs_pp(seed, K)
    xs = [eq1(s, Q, P_PAPER) for s in shingle_strings(text, n, byte_mode)]
    return [min((a[k] * x + b[k]) % P_PAPER for x in xs) if xs else 0xFFFFFFFF for k in range(K)]


# ---- rolling-family mode: every function is Eq. 1 with its own base ----

def bases(seed: int, K: int):
    a, _ = coeffs(seed, K)
    return [257 + x % (P - 257) for x in a]


def signature_rf(text: bytes, n: int, K: int, seed: int = 0, byte_mode: bool = False):
    sh = shingle_strings(text, n, byte_mode)
    return [min(eq1(s, q) % (1 << 32) for s in sh) if sh else 0xFFFFFFFF for q in bases(seed, K)]
