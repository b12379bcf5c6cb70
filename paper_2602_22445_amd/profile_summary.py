"""Helpers for the benchmark's `roofline.traffic` field.

The HBM-traffic summaries under profiles/ end with machine-readable `traffic`
lines (HBM bytes per launch of every kernel, from rocprofv3 FETCH_SIZE /
WRITE_SIZE counter runs) and the hash of the kernel sources they were taken
with; bench.py reports such a figure only while the sources still have that hash.
"""


def source_hash():
    """sha256 over the library's sources (the one the build compiles into the library)."""
    from . import build
    return build.source_hash()


def read_traffic(path):
    """{kernel: bytes per launch} and the source hash of a traffic summary."""
    out, sha = {}, None
    for line in open(path):
        p = line.split()
        if len(p) >= 3 and p[0] == "traffic":
            out[p[1]] = float(dict(q.split("=") for q in p[2:])["hbm_bytes_per_launch"])
        if len(p) == 2 and p[0] == "source_sha256":
            sha = p[1]
    return out, sha
