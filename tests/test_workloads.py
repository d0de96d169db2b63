"""The synthetic workloads have the sizes and structure the five configurations
name (closed forms), are reproducible from their seeds, and keep shared buffers
identical across replicas while per-replica buffers differ."""
import numpy as np

from paper_2202_07848_amd import workloads as wl


def test_config_sizes_closed_form():
    c1 = wl.config(1)
    assert c1.nbytes == 64 * wl.MiB and len(c1.bufs) == 16 and c1.chunk == 4096
    assert sum(not b.shared for b in c1.bufs) == 4
    assert all(256 * wl.KiB <= b.nbytes <= 8 * wl.MiB + 512 for b in c1.bufs[:-1])

    c2 = wl.config(2)
    params = sum(b.nbytes // 2 for b in c2.bufs if b.name.endswith(".param"))
    assert params == 124_439_808                      # GPT-2 small, tied embedding
    assert len(c2.bufs) == 148 * 5 + 1 and c2.chunk == 64 * wl.KiB
    assert c2.nbytes == params * (2 + 12 + 2) + wl.GiB
    assert c2.distinct_bytes == params * 2 + wl.GiB

    c3 = wl.config(3)
    assert len(c3.bufs) == 100_000 and c3.chunk == 4096 and c3.nreplicas == 1
    sizes = np.array([b.nbytes for b in c3.bufs])
    assert sizes.min() >= 512 and sizes.max() <= 2 * wl.MiB and not (sizes % 512).any()
    zero = np.mean([b.kind == "zero" for b in c3.bufs])
    assert 0.19 < zero < 0.21
    assert 23e9 < c3.nbytes < 27e9                    # analytic mean 252 KB x 100 000

    c4 = wl.config(4)
    p4 = sum(b.nbytes // 2 for b in c4.bufs if b.name.endswith(".param"))
    assert 1.30e9 < p4 < 1.33e9 and c4.nreplicas == 4 and c4.chunk == 256 * wl.KiB
    assert sum(b.nbytes for b in c4.bufs if b.name.startswith("act")) == 8 * wl.GiB

    c5 = wl.config(5)
    p5 = sum(b.nbytes // 2 for b in c5.bufs if b.name.endswith(".param"))
    assert abs(p5 - 3.0e9) < 0.03e9 and c5.nreplicas == 2 and c5.chunk == wl.MiB
    assert sum(b.nbytes for b in c5.bufs if b.name.startswith("act")) == 16 * wl.GiB
    assert all(b.nbytes % 512 == 0 for w in (c1, c2, c4, c5) for b in w.bufs)


def test_replicas_share_exactly_the_shared_buffers_and_are_reproducible():
    w = wl.config(2, 12)
    a0, a1, again = wl.numpy_replica(w, 0), wl.numpy_replica(w, 1), wl.numpy_replica(w, 1)
    for spec, x, y, z in zip(w.bufs, a0, a1, again):
        assert x.size == spec.nbytes
        assert np.array_equal(y, z)
        assert np.array_equal(x, y) == spec.shared
    # value distributions: bf16 parameters ~ N(0, 0.02), Adam v >= 0
    i = next(k for k, b in enumerate(w.bufs) if b.name == "wte.param")
    bf = a0[i].view(np.uint16).astype(np.uint32) << 16
    vals = bf.view(np.float32)
    assert abs(float(vals.std()) - 0.02) < 0.002
    j = next(k for k, b in enumerate(w.bufs) if b.name == "wte.adam_v")
    assert float(a0[j].view(np.float32).min()) >= 0.0


def test_dirty_chunk_selection_and_rewrite():
    w = wl.config(3, 500)
    ids = wl.dirty_chunk_ids(w, 0.1, 10)
    assert ids.size == round(0.1 * w.nchunks) and np.all(np.diff(ids) > 0)
    assert np.array_equal(ids, wl.dirty_chunk_ids(w, 0.1, 10))
    t0 = wl.numpy_replica(w, 0)
    t1 = [b.copy() for b in t0]
    wl.numpy_rewrite_chunks(w, t1, ids, 10)
    buf, off, length = wl.chunk_table(w)
    changed = np.array([not np.array_equal(t0[b][o:o + n], t1[b][o:o + n])
                        for b, o, n in zip(buf, off, length)])
    assert np.array_equal(np.flatnonzero(changed), ids)
    assert int(length.sum()) == w.nbytes and buf.size == w.nchunks


def test_arena_layout_is_disjoint_and_aligned():
    for w in (wl.config(1), wl.config(3, 100)):
        offs, total = wl.arena_layout(w)
        sizes = np.array([b.nbytes for b in w.bufs])
        order = np.argsort(offs)
        assert not (offs % 256).any()
        assert np.all(offs[order][1:] >= (offs + sizes)[order][:-1])
        assert (offs + sizes).max() <= total
    w3 = wl.config(3, 100)
    offs, _ = wl.arena_layout(w3)
    assert not np.all(np.diff(offs) > 0)              # placement order differs from list order
