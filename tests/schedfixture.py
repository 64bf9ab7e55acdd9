"""Reader for tests/golden/lvf_worked_example.txt (shared by the oracle pins and
the library's host-logic tests)."""
import os

STATES = {"running": 0, "waiting": 1, "rotary": 2}


def load():
    path = os.path.join(os.path.dirname(__file__), "golden", "lvf_worked_example.txt")
    kv = {}
    for line in open(path):
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=", 1)
            kv[k.strip()] = v.strip()
    params = tuple(float(kv[k]) for k in ("alpha", "beta_b", "beta_f", "slo_tbt", "slo_ttft"))
    reqs = []
    for tok in kv["requests"].split():
        i, st, blk, t = tok.split(":")
        reqs.append((int(i), STATES[st], int(blk), float(t)))
    vlt = [float(x) for x in kv["vlt"].split()]
    cases = []
    for name in ("case_a", "case_b"):
        d = dict(x.split(":") for x in kv[name].split())
        ids = lambda s: [int(x) for x in s.split(",") if x]
        cases.append(dict(b_hbm=int(d["b_hbm"]), b_xfer=int(d["b_xfer"]), preempt=ids(d["preempt"]),
                          prioritize=ids(d["prioritize"]), fcfs=bool(int(d["fcfs"]))))
    return params, reqs, float(kv["t_now"]), vlt, cases
