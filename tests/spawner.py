"""A helper process that starts other programs on request.

The GPU tests run in one Python process that has initialised the GPU long before a test wants
to start a fresh program (the shim test runs an unmodified HIP application under LD_PRELOAD).
Such a process must not fork-and-exec.  This helper is started by tests/conftest.py before
anything has touched the GPU, never touches it itself, and does the starting: one JSON request
per line on stdin ({"argv": [...], "env": {...}, "timeout": seconds}), one JSON reply per line on
stdout ({"rc": int, "stdout": str, "stderr": str}; rc -999 = timed out)."""
import json
import os
import subprocess
import sys


def main() -> int:
    for line in sys.stdin:
        line = line.strip()
        if not line:
            continue
        req = json.loads(line)
        env = dict(os.environ)
        env.update(req.get("env") or {})
        try:
            r = subprocess.run(req["argv"], env=env, capture_output=True, text=True, timeout=req.get("timeout", 60))
            rep = {"rc": r.returncode, "stdout": r.stdout, "stderr": r.stderr}
        except subprocess.TimeoutExpired as e:
            rep = {"rc": -999, "stdout": (e.stdout or b"").decode(errors="replace") if isinstance(e.stdout, bytes) else (e.stdout or ""),
                   "stderr": "timed out"}
        except OSError as e:
            rep = {"rc": -998, "stdout": "", "stderr": str(e)}
        sys.stdout.write(json.dumps(rep) + "\n")
        sys.stdout.flush()
    return 0


if __name__ == "__main__":
    sys.exit(main())
