"""Readers of the cited text fixtures under tests/golden/."""
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def split_structures():
    """(rows, weights) of split_structures.txt: rows = (name, dims, groups per layer, partitions printed),
    weights = (name, largest, smallest number of weight variables printed)."""
    rows, weights = [], []
    with open(os.path.join(GOLDEN, "split_structures.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            parts = [p.strip() for p in line.split(";")]
            if parts[0] == "weights":
                weights.append((parts[1], int(parts[2]), int(parts[3])))
            else:
                rows.append((parts[0], tuple(int(x) for x in parts[1].split("-")),
                             tuple(int(x) for x in parts[2].split("-")), int(parts[3])))
    return rows, weights
