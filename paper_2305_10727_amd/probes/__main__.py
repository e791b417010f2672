import argparse
import os
import subprocess
import sys
import tempfile

HERE = os.path.dirname(os.path.abspath(__file__))
PKG = os.path.dirname(HERE)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default="", help="prefix of the .txt and .json summaries (default: print only)")
    ap.add_argument("--no-gemm", action="store_true", help="skip the section that loops the c1 GEMM through libgpusq")
    a = ap.parse_args()
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not os.path.exists(os.path.join(PKG, "libgpusq.so")):
        sys.exit("libgpusq.so is not built: run `python -m paper_2305_10727_amd.build`")
    with tempfile.TemporaryDirectory(prefix="gpusq_probe_") as tmp:
        exe = os.path.join(tmp, "hw_probes")
        cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               os.path.join(HERE, "hw_probes.hip"), "-o", exe, "-L" + PKG, "-lgpusq", "-Wl,-rpath," + PKG]
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            sys.exit("hipcc failed:\n" + res.stderr)
        run = [exe] + (["--json", a.out + ".json"] if a.out else []) + (["--no-gemm"] if a.no_gemm else [])
        res = subprocess.run(run, capture_output=True, text=True)
        text = "command: python -m paper_2305_10727_amd.probes" + (" --out " + a.out if a.out else "") + "\n\n" + res.stdout
        print(text)
        if res.returncode != 0:
            sys.exit(res.stderr)
        if a.out:
            with open(a.out + ".txt", "w") as fh:
                fh.write(text)


if __name__ == "__main__":
    main()
