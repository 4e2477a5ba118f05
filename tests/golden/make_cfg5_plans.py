"""Writes tests/golden/cfg5_plans.txt: the code-length plans of configuration 5
(100 clients, d = 25.6M, 31 coded groups, a budget of its own per client), each
made by the ORACLE's Algorithm 1 from the exponent the ORACLE fits to that
client's synthetic vector.  Calls nothing but oracle/ and the input generator.
Planning 100 vectors of this size takes minutes of CPU time, which is why the
result is stored; the GPU test that reads the file re-validates every plan.

    python tests/golden/make_cfg5_plans.py
"""
import os
import sys
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import cvlc_synth as syn  # noqa: E402
from oracle import cvlc_oracle as orc  # noqa: E402


def one(client):
    w = syn.WORKLOADS[5]
    U = syn.update_vector(5, client)
    alpha = orc.fit_alpha(U)
    p = orc.plan_for(w, client=client, alpha=alpha)
    return client, alpha, w.budget_bits(client), p.code_len(), p.counts(), int(p.total_bits)


def main():
    w = syn.WORKLOADS[5]
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as ex:
        rows = list(ex.map(one, range(w.n_clients)))
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cfg5_plans.txt")
    with open(path, "w") as f:
        f.write("# Plans of configuration 5, written by tests/golden/make_cfg5_plans.py from the oracle alone\n"
                "# (orc.fit_alpha of cvlc_synth.update_vector(5, client), then orc.plan_alg1 under the client's budget).\n"
                "# client alpha budget_bits total_bits | y_1..y_31 | P_1..P_31\n")
        for client, alpha, budget, y, P, total in rows:
            f.write(f"{client} {alpha!r} {budget} {total} | {' '.join(map(str, y))} | {' '.join(map(str, P))}\n")
    print(path, len(rows), "plans")


if __name__ == "__main__":
    main()
