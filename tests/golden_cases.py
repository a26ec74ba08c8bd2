"""Reader for tests/golden/rne_cases.txt (shared by the oracle pin and the GPU parity test)."""
import os


def load_rne_cases():
    path = os.path.join(os.path.dirname(__file__), "golden", "rne_cases.txt")
    cases = []
    with open(path) as fh:
        for line in fh:
            line = line.split("#", 1)[0].strip()
            if not line:
                continue
            f = line.split()
            cases.append({
                "w": int(f[0], 16), "side": f[1], "gate": float.fromhex(f[2]),
                "b": float.fromhex(f[3]), "a": float.fromhex(f[4]),
                "expect": int(f[5], 16), "tag": f[6] if len(f) > 6 else "",
            })
    return cases
