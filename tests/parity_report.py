"""Formats the achieved errors a GPU run of the parity suite logged (WS_PARITY_LOG=<file>, one JSON object
per case) as a text table:  python tests/parity_report.py <log.jsonl> > profiles/parity_errors.txt
Not collected by pytest (no test_ prefix)."""
import json
import sys

COLS = ["lse_abs", "loss_rel", "row_max_abs", "sumexp_rel", "label_logit_abs", "dX", "dW", "db"]
GATES = {"lse_abs": 2e-3, "loss_rel": 1e-3, "row_max_abs": 2e-3, "sumexp_rel": 1e-3, "label_logit_abs": 2e-3,
         "dX": 2e-2, "dW": 2e-2, "db": 2e-2}


def main(path):
    rows = [json.loads(l) for l in open(path) if l.strip()]
    print("Achieved GPU-vs-oracle errors of the parity suite (one MI355X), written by the tests themselves.")
    print("Command:  WS_PARITY_LOG=parity.jsonl python -m pytest tests -m gpu -x -v")
    print("          python tests/parity_report.py parity.jsonl")
    print("lse / row max / label logit: max absolute error; loss, sum-exp: max relative error per row;")
    print("dX, dW, db: max absolute error relative to the largest magnitude of that gradient.")
    print("Gates: " + "  ".join(f"{k} <= {v:g}" for k, v in GATES.items()))
    print()
    print(f"{'case':58s} " + " ".join(f"{c:>15s}" for c in COLS))
    other = []
    for r in rows:
        if not any(c in r for c in COLS):
            other.append(r)
            continue
        note = ""
        cells = []
        for c in COLS:
            v = r.get(c)
            if c == "loss_rel" and v is not None and v > 1.0:
                cells.append(f"{'(loss~0)':>15s}")           # planted rows whose loss is ~0: gated absolutely
                note = f"  loss_abs={r.get('loss_abs', float('nan')):.1e}"
            else:
                cells.append(f"{v:15.2e}" if v is not None else f"{'-':>15s}")
        print(f"{r['case'][:58]:58s} " + " ".join(cells) + note)
    print()
    for r in other:
        rest = {k: v for k, v in r.items() if k not in ("case", "shape")}
        print(f"{r['case'][:58]:58s} " + "  ".join(f"{k}={v:g}" for k, v in rest.items()))
    print()
    print("Shapes:")
    for r in rows:
        print(f"  {r['case'][:58]:58s} {r['shape']}")


if __name__ == "__main__":
    main(sys.argv[1])
