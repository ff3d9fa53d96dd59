"""Builds libpard.so (hand-written HIP for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB_PATH = os.path.join(HERE, "libpard.so")
HASH_PATH = os.path.join(HERE, "libpard.srchash")
SOURCES = ["pard_api.hip", "pard_fused.hip", "pard_presorted.hip", "pard_sort.hip", "pard_compact.hip", "pard_planner.hip", "pard_ranked.hip", "pard_reactive.hip", "pard_wave.hip"]
HEADERS = ["pard_host.hpp", "pard_device.hpp"]


def _hipcc() -> str:
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def compile_flags():
    return ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
            # packed fp32 instructions are kept out of the generated code on purpose
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-Wall", "-I" + os.path.join(ROOT, "include")]


def hipcc_command(out: str = LIB_PATH):
    """One-line form of the build (every source in one hipcc call)."""
    return [_hipcc(), *compile_flags(), "-shared", *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]


def dependencies():
    return [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", "pard.h")]


def source_hash() -> str:
    """Digest of everything the library is built from (sources, headers, flags)."""
    import hashlib
    h = hashlib.sha256(" ".join(compile_flags()[:-1]).encode())
    for d in dependencies():
        h.update(os.path.basename(d).encode())
        with open(d, "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def is_stale() -> bool:
    """True when the library is missing or was built from other sources than the ones in the tree
    (the digest written next to it at build time no longer matches; file times play no role, so a
    copied tree is judged by its contents)."""
    if not os.path.exists(LIB_PATH) or not os.path.exists(HASH_PATH):
        return True
    with open(HASH_PATH) as f:
        return f.read().strip() != source_hash()


def _filtered(text: str) -> str:
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops' is not a recognized feature" not in l)


def build_library(verbose: bool = False, jobs: int = 8, incremental: bool = False) -> str:
    """Compile every HIP source (one hipcc process per file, side by side) and link them into
    paper_2602_08747_amd/libpard.so.  Recompiles everything unless `incremental`, which keeps
    the objects that are newer than their source and every header."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    digest = source_hash()
    newest_header = max(os.path.getmtime(d) for d in dependencies() if not d.endswith(".hip"))

    def compile_one(src: str):
        obj = os.path.join(OBJ_DIR, os.path.splitext(src)[0] + ".o")
        path = os.path.join(CSRC, src)
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) > max(os.path.getmtime(path), newest_header):
            return src, obj, 0, ""
        cmd = [_hipcc(), *compile_flags(), "-c", path, "-o", obj]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return src, obj, res.returncode, _filtered(res.stdout)

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        results = list(pool.map(compile_one, SOURCES))
    log = "\n".join(out for _, _, _, out in results if out.strip())
    failed = [src for src, _, rc, _ in results if rc != 0]
    if failed:
        raise RuntimeError(f"hipcc failed on {', '.join(failed)}:\n{log}")
    tmp = LIB_PATH + ".tmp"
    res = subprocess.run([_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *[obj for _, obj, _, _ in results], "-o", tmp],
                         stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("linking libpard.so failed:\n" + _filtered(res.stdout))
    os.replace(tmp, LIB_PATH)
    with open(HASH_PATH, "w") as f:
        f.write(digest + "\n")
    if verbose and log.strip():
        print(log, file=sys.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library(verbose=True, incremental="--incremental" in sys.argv))
