"""Host archiver (the last step of Alg. 1): lossless round trip over what the oracle writes, and the
container's own checks.  No GPU."""
import numpy as np
import pytest

import oracle as O
from paper_2406_11257_amd import archive as A

f32 = np.float32


def small(n, seed):
    g = np.random.default_rng(seed)
    Wp = (g.standard_normal(n) * 0.02).astype(f32)
    W = (Wp + g.laplace(0, 1e-4, n).astype(f32)).astype(f32)
    m = (g.standard_normal(n) * 5e-5).astype(f32)
    v = (m.astype(np.float64) ** 2 * g.lognormal(0, 1, n) + 1e-16).astype(f32)
    return Wp, W, m, v


def test_round_trip_of_both_layouts_and_reconstruction():
    entries, want = [], {}
    for i, n in enumerate([0, 1, 1001, 40000]):
        Wp, W, m, v = small(n, i)
        r = O.compress_step(Wp, W, m, v, nbits=4, iters=3)
        head, cw, cm, cv = O.export_dense(r.blob)
        entries.append({"name": f"t{i}.dense", "n": n, "nbits": 4, "layout": "dense",
                        "sections": [head, cw.tobytes(), cm.tobytes(), cv.tobytes()]})
        entries.append({"name": f"t{i}.blob", "n": n, "nbits": 4, "layout": "blob", "sections": [r.blob]})
        want[i] = (Wp, r)
    data = A.pack(entries, preset=6, threads=4)
    back = A.unpack(data, threads=4)
    assert [(e["name"], e["n"], e["nbits"], e["layout"]) for e in back] == \
           [(e["name"], e["n"], e["nbits"], e["layout"]) for e in entries]
    for a, b in zip(entries, back):
        assert [bytes(x) for x in a["sections"]] == b["sections"]
    # what comes out of the archive reconstructs the checkpoint the compressor kept
    for i, (Wp, r) in want.items():
        d = back[2 * i]["sections"]
        n = Wp.size
        Wd, md, vd = O.decompress_dense(Wp, d[0], np.frombuffer(d[1], np.uint8), np.frombuffer(d[2], np.uint8),
                                        np.frombuffer(d[3], np.uint8))
        Wb, mb, vb = O.decompress_step(Wp, back[2 * i + 1]["sections"][0])
        assert Wd.tobytes() == r.W_recon.tobytes() == Wb.tobytes()
        assert md.tobytes() == r.m_recon.tobytes() and vd.tobytes() == r.v_recon.tobytes()
    # the archive is smaller than what went in (the codes of pruned elements repeat)
    raw = sum(len(bytes(s)) for e in entries for s in e["sections"])
    assert len(data) < raw


@pytest.mark.parametrize("codec", ["lzma2", "deflate", "bzip2", "none"])
def test_every_codec_round_trips(codec):
    Wp, W, m, v = small(5000, 3)
    r = O.compress_step(Wp, W, m, v, nbits=4, iters=2)
    head, cw, cm, cv = O.export_dense(r.blob)
    entries = [{"name": "a", "n": 5000, "nbits": 4, "layout": "dense", "sections": [head, cw.tobytes(), cm.tobytes(), cv.tobytes()]},
               {"name": "b", "n": 5000, "nbits": 4, "layout": "blob", "sections": [r.blob]}]
    data = A.pack(entries, preset=2, threads=2, codec=codec)
    back = A.unpack(data, threads=2)
    assert A.read_index(data)[0]["codec"] == codec
    for a, b in zip(entries, back):
        assert [bytes(x) for x in a["sections"]] == b["sections"]
    with pytest.raises(ValueError):
        A.pack(entries, codec="rar")


def test_container_checks():
    e = [{"name": "x", "n": 4, "nbits": 4, "layout": "blob", "sections": [b"abcd" * 100]}]
    data = A.pack(e, preset=1, threads=1)
    index, off = A.read_index(data)
    assert index["tensors"][0]["sections"][0]["raw"] == 400 and data[:8] == b"EXCPARC1"
    with pytest.raises(ValueError):
        A.unpack(b"notanarchive....")
    with pytest.raises(ValueError):
        A.unpack(data[:-3])
    bad = bytearray(data)
    bad[off + 5] ^= 0x40
    with pytest.raises(Exception):
        A.unpack(bytes(bad))
    with pytest.raises(ValueError):
        A.pack([{"name": "x", "n": 4, "nbits": 4, "layout": "dense", "sections": [b""]}])
    with pytest.raises(ValueError):
        A.pack([{"name": "x", "n": 4, "nbits": 4, "layout": "other", "sections": [b""]}])
