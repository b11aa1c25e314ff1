"""Writes hash_vectors.txt: values of the random ranker's counter hash, computed here with Python integers from its
definition (one mixed word per aligned quad of flat element indices, one byte rotation per element; the paper, Sec. III-B,
names no generator).  Run from the repository root: python tests/golden/make_hash_vectors.py"""
import os

M = 0xFFFFFFFF


def hash32(seed, e):
    x, y, s0, s1 = e & M, (e >> 32) & M, seed & M, (seed >> 32) & M
    v = 0xA54FF53A ^ (x >> 2) ^ ((s0 * 0x9E3779B9) & M) ^ ((y * 0xBB67AE85) & M) ^ ((s1 * 0x510E527F) & M)
    v ^= v >> 16
    v = (v * 0x6A09E667) & M
    v ^= v >> 15
    v = (v * 0xBB67AE85) & M
    v ^= v >> 16
    rot = 8 * (x & 3)
    return ((v << rot) | (v >> (32 - rot))) & M & 0xFFFFFFF0   # a key is 28 bits wide: the low four are cleared


CASES = [(0, e) for e in range(16)] + [(1, e) for e in range(8)] + [
    (0, 2 ** 32 - 1), (0, 2 ** 32), (0, 2 ** 32 + 5), (0, 2 ** 40 + 123), (12345, 987654321), (2 ** 32, 7), (2 ** 33 + 12345, 2 ** 32 + 4096),
    (2 ** 63 + 5, 2 ** 35 + 2), (2 ** 64 - 1, 2 ** 40 - 1), (0x1234_5678_9ABC_DEF0, 0xFEDC_BA98_7654_3210 >> 4)]

if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "hash_vectors.txt")
    with open(path, "w") as f:
        f.write("# seed element hash   (decimal seed and element, hexadecimal hash)\n")
        for seed, e in CASES:
            f.write("%d %d 0x%08X\n" % (seed, e, hash32(seed, e)))
    print("wrote", path)
