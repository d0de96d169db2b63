"""Regenerates xxh64_seed0_vectors.txt with the installed xxHash library.

The values pin the CPU oracle to the public XXH64 function, so they must come
from neither the oracle nor the HIP path: this script calls only the
third-party ``xxhash`` package (python-xxhash over libxxhash).  Run it by hand
when vectors are added; the tests read the text file, never this script.

Inputs: "pat n" = first n bytes of b[i] = ((i * 2654435761) mod 2**32) >> 24;
"zeros n" = n zero bytes; "ascii s" = the ASCII bytes of s.  Lengths cover the
short-input path, every tail branch (8-, 4-, 1-byte steps), whole stripes, and
the chunk sizes of the five workloads with their all-zero chunk.
"""
import os
import xxhash

PAT_LENS = [0, 1, 3, 4, 5, 7, 8, 9, 15, 16, 17, 31, 32, 33, 63, 64, 65, 95, 96, 127, 128, 255,
            256, 512, 1536, 4096, 65536, 262144, 1048576]
ZERO_LENS = [512, 4096, 65536, 262144, 1048576]
ASCII = ["a", "abc"]


def pattern(n):
    return bytes((((i * 2654435761) & 0xFFFFFFFF) >> 24) for i in range(n))


def main():
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "xxh64_seed0_vectors.txt")
    with open(out, "w") as f:
        f.write("# XXH64, seed 0, native-integer digest in hex.\n")
        f.write("# Source: xxHash library %s via python-xxhash %s (make_xxh64_vectors.py);\n"
                % (xxhash.XXHASH_VERSION, xxhash.VERSION))
        f.write("# independent of the CPU oracle and of the HIP kernels.  The paper names no\n")
        f.write("# checksum function (sec. 4.6, 5.2.1); XXH64/seed 0 is this build's choice.\n")
        f.write("# kind arg digest\n")
        big = pattern(max(PAT_LENS))
        for n in PAT_LENS:
            f.write("pat %d %016X\n" % (n, xxhash.xxh64_intdigest(big[:n], 0)))
        for n in ZERO_LENS:
            f.write("zeros %d %016X\n" % (n, xxhash.xxh64_intdigest(bytes(n), 0)))
        for s in ASCII:
            f.write("ascii %s %016X\n" % (s, xxhash.xxh64_intdigest(s.encode(), 0)))


if __name__ == "__main__":
    main()
