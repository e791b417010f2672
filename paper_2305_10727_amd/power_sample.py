"""Socket power and shader clocks while one GEMM runs back to back.

    python3 -m paper_2305_10727_amd.power_sample --config c1 --layer fc1 --path int8 --seconds 8 [--out FILE]

Starts `paper_2305_10727_amd.gemm_loop` as a child process with enough launches for the given time, and meanwhile asks
`amd-smi metric -p -c --json` once a second (this process itself never touches the GPU).  Prints, per sample, the socket
power and the clock of every XCD's shader engine domain as the tool reports them, one idle sample first and one after.
"""
import argparse
import json
import subprocess
import sys
import time


def flatten(obj, path=""):
    if isinstance(obj, dict):
        for k, v in obj.items():
            yield from flatten(v, path + "/" + str(k))
    elif isinstance(obj, list):
        for i, v in enumerate(obj):
            yield from flatten(v, path + "/" + str(i))
    else:
        yield path, obj


def sample():
    res = subprocess.run(["amd-smi", "metric", "-p", "-c", "--json"], capture_output=True, text=True)
    if res.returncode != 0:
        return "amd-smi failed: " + (res.stderr.strip().splitlines() or ["?"])[-1]
    try:
        data = json.loads(res.stdout)
    except ValueError:
        return "unparsed: " + " ".join(res.stdout.split())[:400]
    flat = dict(flatten(data))
    power = [(p, v) for p, v in flat.items() if "socket_power" in p and p.endswith("/value")]
    clocks = [(p, v) for p, v in flat.items() if "/gfx_" in p and p.endswith("/clk/value")]
    if not power and not clocks:  # another layout of the tool's output: keep what names power or a gfx clock
        keep = [(p, v) for p, v in flat.items() if ("power" in p or "gfx" in p) and isinstance(v, (int, float))]
        return " ".join("%s=%s" % (p, v) for p, v in keep[:24])
    return "socket_power_W=%s gfx_clk_MHz=%s" % ("/".join(str(v) for _, v in power), " ".join(str(v) for _, v in clocks))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", default="c1")
    ap.add_argument("--layer", default="fc1")
    ap.add_argument("--path", default="int8", choices=["int8", "fp16"])
    ap.add_argument("--kind", default="sparse", choices=["sparse", "dense"])
    ap.add_argument("--seconds", type=float, default=8.0)
    ap.add_argument("--us-per-launch", type=float, default=40.0, help="rough launch time, to size the child's loop")
    ap.add_argument("--out", default="")
    a = ap.parse_args()
    lines = ["command: python3 -m paper_2305_10727_amd.power_sample " + " ".join(sys.argv[1:]), "", "idle before: " + sample()]
    iters = int(a.seconds * 1e6 / a.us_per_launch)
    child = subprocess.Popen([sys.executable, "-m", "paper_2305_10727_amd.gemm_loop", "--config", a.config, "--layer", a.layer,
                              "--path", a.path, "--kind", a.kind, "--iters", str(iters)], stdout=subprocess.PIPE, text=True)
    t0 = time.time()
    time.sleep(1.0)
    while child.poll() is None and time.time() - t0 < a.seconds + 120:
        lines.append("t=%5.1f s: %s" % (time.time() - t0, sample()))
        print(lines[-1], flush=True)
        time.sleep(1.0)
    out, _ = child.communicate(timeout=60)
    lines.append("child: " + out.strip())
    time.sleep(2.0)
    lines.append("idle after: " + sample())
    text = "\n".join(lines) + "\n"
    print(text)
    if a.out:
        with open(a.out, "w") as fh:
            fh.write(text)
    return child.returncode


if __name__ == "__main__":
    sys.exit(main())
