"""Builds libtri.so (the HIP kernels and the C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libtri.so")
SOURCES = ["tri_api.hip", "tri_centers.hip", "tri_score.hip", "tri_score_mfma.hip", "tri_score_lane.hip", "tri_select.hip", "tri_compact.hip"]

# packed fp32 VALU forms are switched off for every kernel of this library
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc():
    return os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build(verbose=False, extra=()):
    """Compile every .hip source (in parallel, one hipcc process each) and link libtri.so.  Always recompiles."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    def clean(text):   # hipcc's host pass does not know the packed-fp32 feature name and says so: harmless
        return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l)

    with tempfile.TemporaryDirectory(prefix="libtri_build_") as tmp:
        def compile_one(src):
            obj = os.path.join(tmp, src.replace(".hip", ".o"))
            cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-c", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                   os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
            return src, obj, res.returncode, clean(res.stdout)

        with ThreadPoolExecutor(max_workers=min(len(SOURCES), os.cpu_count() or 1)) as ex:
            results = list(ex.map(compile_one, SOURCES))
        for src, _, rc, out in results:
            if rc != 0:
                raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
            if verbose and out.strip():
                print(out)
        cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", *[r[1] for r in results], "-o", LIB]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + clean(res.stdout))
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
