"""The CPU oracle over many tensors at once, for the full-size GPU parity tests and the benchmark's
CPU-baseline leg.  TEST INFRASTRUCTURE ONLY, like the rest of this package.

The oracle is single-threaded numpy; a checkpoint-sized comparison fans its tensors out over the host's
cores.  Workers are separate interpreter processes started from this file (`python pool.py
--worker DIR`): they import numpy and the oracle only -- nothing of the HIP library, no torch, and they
never see the GPU.  Work travels through a scratch directory (memory-backed when /dev/shm exists): the
parent writes a tensor's inputs as .npy files, copied from what the GPU was given so that both sides
read the same bytes, then a task file; a worker claims a task by renaming it (atomic), runs the oracle
and leaves a result file.  Larger tensors are taken first.
"""
from __future__ import annotations

import hashlib
import json
import os
import pickle
import shutil
import subprocess
import sys
import tempfile
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FIELDS = ("Wp", "W", "m", "v")


def workers() -> int:
    """Worker processes: the host's share of cores, 16 at most."""
    try:
        have = len(os.sched_getaffinity(0))
    except AttributeError:
        have = os.cpu_count() or 1
    return max(1, min(16, have))


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).view(np.uint8)).hexdigest()


def run_task(directory: str, task: dict) -> dict:
    """One tensor through the oracle."""
    import oracle as O
    key, params = task["key"], task["params"]
    arrs = [np.load(os.path.join(directory, f"{key}_{f}.npy"), mmap_mode="r") for f in FIELDS]
    t0 = time.time()
    ref = O.compress_step(*arrs, params["alpha"], params["beta"], params["nbits"], params["iters"],
                          flags=params.get("flags", 0))
    out = dict(key=key, n=ref.n, n_w=ref.n_w, n_o=ref.n_o, nbytes=len(ref.blob),
               blob_sha=hashlib.sha256(ref.blob).hexdigest(),
               median=np.float32(ref.median).tobytes(), mean=np.float32(ref.mean_abs_m).tobytes(),
               t_w=np.float32(ref.t_w).tobytes(), r_o=np.float32(ref.r_o).tobytes(), abs_sum_m=float(ref.abs_sum_m),
               W_sha=digest(ref.W_recon), m_sha=digest(ref.m_recon), v_sha=digest(ref.v_recon),
               books={k: np.asarray(c, dtype=np.float32).tobytes() for k, c in ref.C.items()},
               obj={k: float(x) for k, x in ref.obj.items()}, seconds=time.time() - t0)
    if task.get("want_blob"):
        out["blob"] = ref.blob
    return out


def worker_main(directory: str) -> None:
    sys.path.insert(0, ROOT)
    while True:
        names = sorted(n for n in os.listdir(directory) if n.startswith("task_"))
        claimed = None
        for name in names:
            mine = os.path.join(directory, "run_" + name[5:])
            try:
                os.rename(os.path.join(directory, name), mine)
                claimed = mine
                break
            except OSError:
                continue                         # another worker took it
        if claimed is None:
            if os.path.exists(os.path.join(directory, "stop")):
                return
            time.sleep(0.05)
            continue
        with open(claimed) as f:
            task = json.load(f)
        try:
            res = run_task(directory, task)
        except Exception as e:                   # reported to the parent, which fails the test
            res = dict(key=task["key"], error=repr(e))
        tmp = os.path.join(directory, "tmp_" + task["key"])
        with open(tmp, "wb") as f:
            pickle.dump(res, f)
        os.rename(tmp, os.path.join(directory, "res_" + task["key"]))
        os.remove(claimed)


class OraclePool:
    """with OraclePool() as pool: pool.submit(key, (Wp, W, m, v), params) ...; pool.result(key) ..."""

    def __init__(self, nworkers: int | None = None):
        base = "/dev/shm" if os.path.isdir("/dev/shm") and os.access("/dev/shm", os.W_OK) else None
        self.dir = tempfile.mkdtemp(prefix="excp_oracle_", dir=base)
        env = dict(os.environ, OMP_NUM_THREADS="1", OPENBLAS_NUM_THREADS="1", MKL_NUM_THREADS="1",
                   HIP_VISIBLE_DEVICES="", CUDA_VISIBLE_DEVICES="")
        self.procs = [subprocess.Popen([sys.executable, "-u", os.path.abspath(__file__), "--worker", self.dir], env=env)
                      for _ in range(nworkers or workers())]
        self.keys = []

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()
        return False

    def close(self):
        if self.procs:
            open(os.path.join(self.dir, "stop"), "w").close()
            for name in os.listdir(self.dir):                        # nothing more is wanted: unclaimed tasks go
                if name.startswith("task_"):
                    try:
                        os.remove(os.path.join(self.dir, name))
                    except OSError:
                        pass
            for p in self.procs:
                try:
                    p.wait(timeout=600)
                except subprocess.TimeoutExpired:
                    p.kill()
            self.procs = []
        shutil.rmtree(self.dir, ignore_errors=True)

    def submit(self, key: str, arrays, params: dict, want_blob: bool = False):
        n = int(np.asarray(arrays[1]).size)
        for f, a in zip(FIELDS, arrays):
            np.save(os.path.join(self.dir, f"{key}_{f}.npy"), np.ascontiguousarray(a))
        tmp = os.path.join(self.dir, "new_" + key)
        with open(tmp, "w") as f:
            json.dump(dict(key=key, params=params, want_blob=want_blob), f)
        os.rename(tmp, os.path.join(self.dir, f"task_{10**12 - n:013d}_{key}"))     # larger tensors sort first
        self.keys.append(key)

    def outstanding(self) -> int:
        return sum(1 for k in self.keys if not os.path.exists(os.path.join(self.dir, "res_" + k)))

    def result(self, key: str, timeout: float = 900.0) -> dict:
        path = os.path.join(self.dir, "res_" + key)
        t0 = time.time()
        while not os.path.exists(path):
            if any(p.poll() not in (None, 0) for p in self.procs):
                raise RuntimeError("an oracle worker died")
            if time.time() - t0 > timeout:
                raise TimeoutError(f"oracle result {key}")
            time.sleep(0.02)
        with open(path, "rb") as f:
            res = pickle.load(f)
        os.remove(path)
        for f in FIELDS:
            try:
                os.remove(os.path.join(self.dir, f"{key}_{f}.npy"))
            except OSError:
                pass
        self.keys.remove(key)
        if "error" in res:
            raise RuntimeError(f"oracle failed on {key}: {res['error']}")
        return res


if __name__ == "__main__":
    if len(sys.argv) == 3 and sys.argv[1] == "--worker":
        worker_main(sys.argv[2])
