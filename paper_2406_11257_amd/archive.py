"""Host side of the last step of Alg. 1: a general-purpose lossless archiver over what the GPU wrote.

The paper packs the code tensors and codebooks with 7zip (LZMA2, "ultra"; Sec. 4.2 and Table
"compact").  This module does the same with liblzma (the LZMA2 filter, preset 9 extreme) through
Python's ``lzma``; everything before it -- the codes, the per-element layout of Sec. 4.2 -- comes
from the HIP library.  Nothing here computes any part of the method; it only moves bytes.

Archive file (little endian):
    8 B   magic "EXCPARC1"
    8 B   u64 length L of the index
    L B   index, UTF-8 JSON: {"tensors": [{"name", "n", "nbits", "layout", "sections":
          [{"raw", "packed", "crc"} ...]} ...], "preset", "codec"}
    ...   the packed sections, back to back, in index order; each one is a raw LZMA2 stream (or, for
          the comparison of Table "compact", a zlib or bzip2 stream)

Layouts: "dense" = head, codes_w, codes_m, codes_v (the paper's stored layout, one code per
element); "blob" = the compressed tensor of the C ABI as one section (bitmaps + packed codes).
Sections are packed independently so that a thread pool can work on them (liblzma releases the
interpreter lock) and a single tensor can be read back without the others.
"""
from __future__ import annotations

import bz2
import json
import lzma
import struct
import zlib
from concurrent.futures import ThreadPoolExecutor

MAGIC = b"EXCPARC1"
DEFAULT_PRESET = 9 | lzma.PRESET_EXTREME
CODECS = ("lzma2", "deflate", "bzip2", "none")      # Table "compact" compares 7z with zip and bz2


def _filters(preset: int):
    return [{"id": lzma.FILTER_LZMA2, "preset": preset}]


def _encode(raw: bytes, codec: str, preset: int) -> bytes:
    if codec == "lzma2":
        return lzma.compress(raw, format=lzma.FORMAT_RAW, filters=_filters(preset))
    if codec == "deflate":
        return zlib.compress(raw, 9)
    if codec == "bzip2":
        return bz2.compress(raw, 9)
    if codec == "none":
        return raw
    raise ValueError("unknown codec " + codec)


def _decode(packed: bytes, codec: str, preset: int) -> bytes:
    if codec == "lzma2":
        return lzma.decompress(packed, format=lzma.FORMAT_RAW, filters=_filters(preset))
    if codec == "deflate":
        return zlib.decompress(packed)
    if codec == "bzip2":
        return bz2.decompress(packed)
    if codec == "none":
        return packed
    raise ValueError("unknown codec " + codec)


def pack(tensors, preset: int = DEFAULT_PRESET, threads: int = 8, codec: str = "lzma2") -> bytes:
    """tensors: sequence of dicts {"name", "n", "nbits", "layout", "sections": [bytes-like, ...]}.
    codec: "lzma2" (the paper's choice), "deflate", "bzip2" or "none".  Returns the archive."""
    if codec not in CODECS:
        raise ValueError("unknown codec " + str(codec))
    jobs = []
    for t in tensors:
        if t["layout"] not in ("dense", "blob"):
            raise ValueError("unknown layout " + str(t["layout"]))
        if t["layout"] == "dense" and len(t["sections"]) != 4:
            raise ValueError("the dense layout has four sections: head, codes_w, codes_m, codes_v")
        for s in t["sections"]:
            jobs.append((bytes(s), preset))
    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        packed = list(pool.map(lambda job: _encode(job[0], codec, job[1]), jobs))
    index, k = {"preset": preset, "codec": codec, "tensors": []}, 0
    for t in tensors:
        secs = []
        for s in t["sections"]:
            raw = jobs[k][0]
            secs.append({"raw": len(raw), "packed": len(packed[k]), "crc": zlib.crc32(raw)})
            k += 1
        index["tensors"].append({"name": t["name"], "n": int(t["n"]), "nbits": int(t["nbits"]),
                                 "layout": t["layout"], "sections": secs})
    idx = json.dumps(index, separators=(",", ":")).encode()
    return MAGIC + struct.pack("<Q", len(idx)) + idx + b"".join(packed)


def read_index(data: bytes) -> tuple[dict, int]:
    """The index of an archive and the offset of its first packed section."""
    if len(data) < 16 or data[:8] != MAGIC:
        raise ValueError("not an ExCP archive")
    (length,) = struct.unpack("<Q", data[8:16])
    if 16 + length > len(data):
        raise ValueError("truncated index")
    return json.loads(data[16:16 + length].decode()), 16 + length


def unpack(data: bytes, threads: int = 8):
    """Inverse of pack(): the list of tensors with their raw sections (bytes); verifies lengths and CRCs."""
    index, off = read_index(data)
    preset, codec = index["preset"], index.get("codec", "lzma2")
    if codec not in CODECS:
        raise ValueError("unknown codec " + str(codec))
    jobs = []
    for t in index["tensors"]:
        for s in t["sections"]:
            if off + s["packed"] > len(data):
                raise ValueError("truncated archive")
            jobs.append((data[off:off + s["packed"]], s))
            off += s["packed"]

    def one(job):
        blob, s = job
        raw = _decode(blob, codec, preset)
        if len(raw) != s["raw"] or zlib.crc32(raw) != s["crc"]:
            raise ValueError("a section does not match its index entry")
        return raw

    with ThreadPoolExecutor(max_workers=max(1, threads)) as pool:
        raws = list(pool.map(one, jobs))
    out, k = [], 0
    for t in index["tensors"]:
        cnt = len(t["sections"])
        out.append({"name": t["name"], "n": t["n"], "nbits": t["nbits"], "layout": t["layout"],
                    "sections": raws[k:k + cnt]})
        k += cnt
    return out


# ---------------------------------------------------------------------------------------------
# GPU <-> archive.  `ctx` is a paper_2406_11257_amd.Context; blobs are what its compress calls wrote.
# ---------------------------------------------------------------------------------------------
def save_checkpoint(ctx, named_blobs, nbits: int, layout: str = "dense", preset: int = DEFAULT_PRESET,
                    threads: int = 8, codec: str = "lzma2") -> bytes:
    """named_blobs: sequence of (name, blob device tensor, blob_bytes, n).  Exports the paper's stored
    layout on the GPU (layout "dense") or takes the blobs as they are ("blob"), copies to the host
    and packs.  Returns the archive bytes."""
    import torch
    from . import binding as B

    tensors = []
    if layout == "dense":
        hb = B.excp_head_bytes(nbits)
        items, bufs = [], []
        for (name, blob, nbytes, n) in named_blobs:
            db = B.excp_dense_bytes(n, nbits)
            b = [torch.empty(max(x, 16), dtype=torch.uint8, device=blob.device) for x in (hb, db, db, db)]
            bufs.append((b, (hb, db, db, db)))
            items.append((blob, nbytes, n, *b))
        ctx.excp_export_dense(items)
        ctx.excp_collect()
        for (name, blob, nbytes, n), (b, sizes) in zip(named_blobs, bufs):
            secs = [t[:s].cpu().numpy().tobytes() for t, s in zip(b, sizes)]
            tensors.append({"name": name, "n": n, "nbits": nbits, "layout": "dense", "sections": secs})
    elif layout == "blob":
        for (name, blob, nbytes, n) in named_blobs:
            tensors.append({"name": name, "n": n, "nbits": nbits, "layout": "blob",
                            "sections": [blob[:nbytes].cpu().numpy().tobytes()]})
    else:
        raise ValueError("unknown layout " + layout)
    return pack(tensors, preset, threads, codec)


def load_checkpoint(ctx, data: bytes, W_prev, want_moments: bool = True, threads: int = 8):
    """Inverse of save_checkpoint: W_prev maps tensor name -> previous reconstructed weights (device;
    fp32, or fp16 / bf16 if the checkpoint was compressed from such weights).  Returns name -> (W_hat, m_hat, v_hat) device tensors (moments None unless wanted)."""
    import numpy as np
    import torch
    from . import binding as B

    entries = unpack(data, threads)
    dense, blobs, keep, out = [], [], [], {}
    for e in entries:
        Wp = W_prev[e["name"]]
        n = e["n"]
        dev = []
        for sec in e["sections"]:
            padded = bytes(sec) + b"\0" * (max(16, (len(sec) + 15) // 16 * 16) - len(sec))
            dev.append(torch.from_numpy(np.frombuffer(padded, dtype=np.uint8).copy()).to(Wp.device))
        keep.append(dev)
        W = torch.empty(n, dtype=Wp.dtype, device=Wp.device)        # the storage the blob was written for
        m = torch.empty(n, dtype=torch.float32, device=Wp.device) if want_moments else None
        v = torch.empty(n, dtype=torch.float32, device=Wp.device) if want_moments else None
        out[e["name"]] = (W, m, v)
        if e["layout"] == "dense":
            dense.append((Wp, dev[0], len(e["sections"][0]), n, dev[1], dev[2] if want_moments else None,
                          dev[3] if want_moments else None, W, m, v))
        else:
            blobs.append((Wp, dev[0], len(e["sections"][0]), n, W, m, v))
    if dense:
        ctx.excp_decompress_dense(dense)
        ctx.excp_collect()
    if blobs:
        ctx.excp_decompress_tensors(blobs)
        ctx.excp_collect()
    return out


def _report(cid: int, preset: int, threads: int, max_tensors: int | None) -> None:
    """Compress one synthetic checkpoint on the GPU and print the sizes of every stage (context for
    the paper's storage tables; the synthetic inputs carry none of a real checkpoint's structure)."""
    import time
    import torch
    from . import binding as B
    from . import synth

    cfg = synth.config(cid)
    specs = list(enumerate(cfg.tensors))[:max_tensors]
    max_n = max(s.n for _, s in specs)
    total = sum(s.n for _, s in specs)
    ctx = B.Context(max_n, min(total, max(max_n, 1 << 28)))
    dev = torch.device("cuda:0")
    tens, named = [], []
    for idx, spec in specs:
        Wp, W, m, v = synth.torch_draw_tensor(cid, idx, spec, dev)
        blob = torch.empty(B.excp_blob_bound(spec.n, synth.NBITS), dtype=torch.uint8, device=dev)
        tens.append((Wp, W, m, v, blob, None))
    ctx.excp_compress_tensors(tens, synth.ALPHA, synth.BETA, synth.NBITS, synth.LLOYD_ITERS, 0)
    rc, stats = ctx.excp_collect()
    for (idx, spec), t, st in zip(specs, tens, stats):
        named.append((spec.name, t[4], int(st.blob_bytes), spec.n))
    raw = 12 * total
    blob_bytes = sum(x[2] for x in named)
    dense_bytes = sum(B.excp_head_bytes(synth.NBITS) + 3 * B.excp_dense_bytes(n, synth.NBITS) for (_, _, _, n) in named)
    print(f"{cfg.name}: {len(named)} tensors, {total} parameters, fp32 W+m+v {raw} B")
    print(f"  kept: weights {sum(s.n_w for s in stats) / total:.4f}, moments {sum(s.n_o for s in stats) / total:.4f}")
    print(f"  blob (bitmaps + packed codes): {blob_bytes} B  ratio {raw / blob_bytes:.2f}")
    print(f"  per-element codes (Sec. 4.2):   {dense_bytes} B  ratio {raw / dense_bytes:.2f}")
    for layout in ("dense", "blob"):
        for codec in ("lzma2", "bzip2", "deflate"):
            t0 = time.time()
            data = save_checkpoint(ctx, named, synth.NBITS, layout=layout, preset=preset, threads=threads, codec=codec)
            dt = time.time() - t0
            how = f"LZMA2 (preset {preset & 15}{'e' if preset & lzma.PRESET_EXTREME else ''})" if codec == "lzma2" else codec
            print(f"  {layout:5s} + {how}, {threads} threads: {len(data)} B  ratio {raw / len(data):.2f}  ({dt:.1f} s)", flush=True)
    ctx.close()


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="sizes of one synthetic compressed checkpoint after every stage")
    ap.add_argument("--config", type=int, default=0)
    ap.add_argument("--preset", type=int, default=9)
    ap.add_argument("--extreme", action="store_true")
    ap.add_argument("--threads", type=int, default=16)
    ap.add_argument("--max-tensors", type=int, default=None)
    a = ap.parse_args()
    _report(a.config, a.preset | (lzma.PRESET_EXTREME if a.extreme else 0), a.threads, a.max_tensors)
