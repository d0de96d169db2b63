"""Are the oracle's pins sharp?  Each case plants one plausible mistake in a
copy of ckpt_oracle.c (a wrong rotate, a swapped prime, a transposed lane, a
dropped term, an off-by-one bound, a wrong offset...), builds it on the CPU and
requires that at least one pin fails.  The pins used here are the ones that do
not depend on the oracle: stored XXH64 vectors, NumPy closed forms, brute-force
byte comparison, round trips."""
import os
import subprocess
import sys

import pytest

import oracle

SRC = os.path.join(os.path.dirname(oracle.__file__), "ckpt_oracle.c")

MUTATIONS = [
    # (name, old text, new text) -- old must occur exactly once
    ("round rotate 31->30", "acc = rotl64(acc, 31);", "acc = rotl64(acc, 30);"),
    ("round primes swapped", "acc += word * P2;\n  acc = rotl64(acc, 31);\n  return acc * P1;",
     "acc += word * P1;\n  acc = rotl64(acc, 31);\n  return acc * P2;"),
    ("v1 init drops P2", "uint64_t v1 = seed + P1 + P2;", "uint64_t v1 = seed + P1;"),
    ("v4 init sign", "uint64_t v4 = seed - P1;", "uint64_t v4 = seed + P1;"),
    ("lanes 2 and 3 transposed", "v2 = xxh_round(v2, le64(p + 8));\n      v3 = xxh_round(v3, le64(p + 16));",
     "v2 = xxh_round(v2, le64(p + 16));\n      v3 = xxh_round(v3, le64(p + 8));"),
    ("converge rotate 18->17", "rotl64(v4, 18)", "rotl64(v4, 17)"),
    ("merge order v2/v3", "h = xxh_merge(h, v2);\n    h = xxh_merge(h, v3);",
     "h = xxh_merge(h, v3);\n    h = xxh_merge(h, v2);"),
    ("merge adds P3 instead of P4", "return h * P1 + P4;", "return h * P1 + P3;"),
    ("length not added", "  h += len;\n", "  /* h += len; */\n"),
    ("stripe loop off by one", "while (left >= 32) {", "while (left > 32) {"),
    ("short-input threshold", "if (len >= 32) {", "if (len > 32) {"),
    ("tail8 rotate", "h = rotl64(h, 27) * P1 + P4;", "h = rotl64(h, 26) * P1 + P4;"),
    ("tail4 rotate", "h = rotl64(h, 23) * P2 + P3;", "h = rotl64(h, 22) * P2 + P3;"),
    ("tail4 multiplier", "h ^= le32(p) * P1;", "h ^= le32(p) * P2;"),
    ("tail1 rotate", "h = rotl64(h, 11) * P1;", "h = rotl64(h, 12) * P1;"),
    ("tail1 prime", "h ^= (uint64_t)(*p) * P5;", "h ^= (uint64_t)(*p) * P1;"),
    ("avalanche shift 33", "h ^= h >> 33;", "h ^= h >> 32;"),
    ("avalanche shift 29", "h ^= h >> 29;", "h ^= h >> 28;"),
    ("avalanche last shift", "h ^= h >> 32;\n  return h;", "h ^= h >> 31;\n  return h;"),
    ("avalanche primes swapped", "h *= P2;\n  h ^= h >> 29;\n  h *= P3;", "h *= P3;\n  h ^= h >> 29;\n  h *= P2;"),
    ("big-endian word read", "for (int i = 7; i >= 0; --i) v = (v << 8) | p[i];",
     "for (int i = 0; i < 8; ++i) v = (v << 8) | p[i];"),
    ("pad to 8 instead of 16", "return (x + 15) & ~(uint64_t)15;", "return (x + 7) & ~(uint64_t)7;"),
    ("ceil division dropped", "return nbytes / chunk + (nbytes % chunk != 0);", "return nbytes / chunk;"),
    ("diff sense inverted", "(ref == NULL || dig[k] != ref[k]) ? 1 : 0", "(ref == NULL || dig[k] == ref[k]) ? 1 : 0"),
    ("compact offsets unpadded", "      e += 1;\n      soff += padded;", "      e += 1;\n      soff += len;"),
    ("manifest offset in chunks", "manifest[e].buf_off = off;", "manifest[e].buf_off = j;"),
    ("manifest digest of wrong chunk", "manifest[e].digest = dig[k];", "manifest[e].digest = dig[e];"),
    ("padding not zeroed", "memset(out + soff + len, 0, padded - len);", "(void)0;"),
    ("restore copies padded length", "in + m->stage_off, m->len);", "in + m->stage_off, (m->len + 15) & ~15u);"),
    ("restore to wrong offset", "(uint8_t *)dst[m->buf].ptr + m->buf_off, in", "(uint8_t *)dst[m->buf].ptr + m->stage_off, in"),
    ("thread split loses the boundary chunk", "if (k < job->k_lo || k >= job->k_hi) continue;",
     "if (k <= job->k_lo || k >= job->k_hi) continue;"),
    ("match: same position not preferred", "if (k < n_ref && ref[k] == dig[k]) {", "if (0) {"),
    ("match: highest reference position taken", "if (pairs[mid].dig < d) lo = mid + 1; else hi = mid;",
     "if (pairs[mid].dig <= d && !(pairs[mid].dig == d && mid + 1 < n && pairs[mid + 1].dig != d) && !(pairs[mid].dig == d && mid + 1 == n)) lo = mid + 1; else hi = mid;"),
    ("match: first occurrence taken for its own duplicate", "if ((uint64_t)k0 < k) {",
     "if ((uint64_t)k0 <= k) {"),
    ("match: duplicate encoding off by one", "s = -2 - k0;", "s = -1 - k0;"),
    ("match: moved chunks also staged", "counts->nmoved += 1;", "counts->nmoved += 1; counts->staged_bytes += 16;"),
    ("match: mask set for duplicates", "mask[k] = (s == -1) ? 1 : 0;", "mask[k] = (s < 0) ? 1 : 0;"),
    ("apply: duplicates before reference copies", "if (s == -1 || (pass == 0) != (s >= 0)) continue;",
     "if (s == -1 || (pass == 1) != (s >= 0)) continue;"),
    ("apply: length mismatch accepted", "if (!ok || flen != tlen) {", "if (!ok) {"),
    ("validate: new checksums not compared", "if (ca != cb || (ca && after_a[k] != after_b[k])) {",
     "if (ca != cb) {"),
    ("validate: change of b read from a", "int cb = before_b[k] != after_b[k];", "int cb = before_a[k] != after_b[k];"),
    ("validate: last mismatch reported", "if (first == ~(uint64_t)0) first = k;", "first = k;"),
    ("owner: lowest rank always uploads", "(k % size == my_place) ? 1 : 0", "(0 == my_place) ? 1 : 0"),
    ("owner: group taken against rank 0", "uint64_t mine = gathered[(uint64_t)rank * N + k];",
     "uint64_t mine = gathered[k];"),
    ("owner: place counted after the increment", "if (r == rank) my_place = size;\n        size += 1;",
     "size += 1;\n        if (r == rank) my_place = size;"),
    ("owner: rotation by rank count instead of group size", "(k % size == my_place)",
     "(k % world == my_place)"),
    ("chain: the first link that holds a chunk wins",
     "memcpy((uint8_t *)dst[t->buf].ptr + t->buf_off, from + t->stage_off, t->len);",
     "if (!written[base[t->buf] + t->buf_off / chunk]) memcpy((uint8_t *)dst[t->buf].ptr + t->buf_off, from + t->stage_off, t->len);"),
    ("chain: shortened chunks accepted", "ok = t->len == (left < chunk ? left : chunk);",
     "ok = t->len <= (left < chunk ? left : chunk);"),
    ("chain: offsets inside a chunk accepted", "t->buf_off % chunk == 0;", "t->buf_off % 16 == 0;"),
    ("chain: staging bound taken from the first link",
     "t->len <= links[l].staging_bytes - t->stage_off;", "t->len <= links[0].staging_bytes - t->stage_off;"),
    ("chain: chunk id without the buffer's base", "uint64_t k = base[t->buf] + t->buf_off / chunk;",
     "uint64_t k = t->buf_off / chunk;"),
    ("chain: every applied entry counted as superseded", "stats[1] = applied - distinct;",
     "stats[1] = applied;"),
    ("chain: skipped entries not counted",
     "        skipped += 1;\n        continue;\n      }\n      uint64_t k = base[t->buf]",
     "        continue;\n      }\n      uint64_t k = base[t->buf]"),
    ("chain: restriction ignored", "      if (only && !only[k]) continue;", "      (void)only;"),
    ("chain: restriction inverted", "      if (only && !only[k]) continue;",
     "      if (only && only[k]) continue;"),
    ("chain: restriction looked up by entry index", "      if (only && !only[k]) continue;",
     "      if (only && !only[e]) continue;"),
    ("merge: entry of the first holder, bytes of the last", "      holder[k] = c;\n",
     "      if (!holder[k]) holder[k] = c;\n"),
    ("merge: bytes taken from the first link's staging",
     "bytes_of[k] = (const uint8_t *)links[l].staging + c->stage_off;",
     "bytes_of[k] = (const uint8_t *)links[0].staging + c->stage_off;"),
    ("merge: entry keeps its old staging offset", "manifest[made].stage_off = at;", "(void)0;"),
    ("merge: offsets unpadded", "    at += slot;\n", "    at += width;\n"),
    ("merge: padding not zeroed", "memset(merged + at + width, 0, slot - width);", "(void)0;"),
    ("merge: staging capacity ignored in the overflow count",
     "int bytes_fit = entry_fits && at + slot <= staging_cap;",
     "int bytes_fit = entry_fits && at <= staging_cap;"),
    ("merge: shortened chunks accepted", "ok = c->len == (rest < chunk ? rest : chunk);",
     "ok = c->len <= (rest < chunk ? rest : chunk);"),
    ("verdicts: only the first chunk of a buffer looked at", "      if (mask[k]) any = 1;",
     "      if (mask[k] && j == 0) any = 1;"),
    ("verdicts: chunk counter not advanced over clean buffers",
     "    for (uint64_t j = 0; j < n; ++j, ++k)\n      if (mask[k]) any = 1;",
     "    for (uint64_t j = 0; j < n; ++j) {\n      if (mask[k]) any = 1;\n      if (any) ++k;\n    }"),
    ("verdicts: bytes counted in chunks", "      bytes += sizes[i];", "      bytes += n * chunk;"),
    ("marks: flag of the wrong buffer", "marks[k++] = flags[i] ? 1 : 0;", "marks[k++] = flags[j < nbufs ? j : i] ? 1 : 0;"),
    ("marks: flag value copied instead of 0 / 1", "marks[k++] = flags[i] ? 1 : 0;", "marks[k++] = flags[i];"),
    ("andnot: second mask not negated", "(mask[k] != 0 && without[k] == 0) ? 1 : 0",
     "(mask[k] != 0 && without[k] != 0) ? 1 : 0"),
    ("andnot: only the value 1 counts as set", "(mask[k] != 0 && without[k] == 0) ? 1 : 0",
     "(mask[k] == 1 && without[k] == 0) ? 1 : 0"),
    ("owner: row stride of gathered checksums", "if (gathered[(uint64_t)r * N + k] != mine) continue;",
     "if (gathered[(uint64_t)r * (N - 1) + k] != mine) continue;"),
]


PINS = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_pins.py")


def run_pins(lib=None) -> int:
    cmd = [sys.executable, PINS] + ([str(lib)] if lib else [])
    return subprocess.run(cmd, stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL).returncode


def test_pins_hold_for_the_real_oracle():
    pytest.importorskip("xxhash")
    assert run_pins() == 0


@pytest.mark.parametrize("name,old,new", MUTATIONS, ids=[m[0] for m in MUTATIONS])
def test_planted_mistake_is_caught(name, old, new, tmp_path):
    pytest.importorskip("xxhash")
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not unique"
    src = tmp_path / "mutant.c"
    lib = tmp_path / "libmutant.so"
    src.write_text(text.replace(old, new))
    subprocess.run(["gcc", "-O1", "-std=c11", "-w", "-fPIC", "-shared", "-pthread", str(src), "-o",
                    str(lib)], check=True)
    # exit 1 = a pin failed; a negative code = the mistake crashed the child: caught either way
    assert run_pins(lib) != 0, f"no pin notices: {name}"
