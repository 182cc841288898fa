"""Parser for the hand-derived mask fixtures under tests/golden/ (plain text, no code)."""
import glob
import os

import numpy as np

CLASS_ID = {"dense": 0, "sink": 1, "intra": 2, "intra_sink": 3}


def load(path):
    runs, sink_len, masks, cur = None, 0, {}, None
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("runs:"):
                runs = []
                for tok in line[5:].split():
                    kind = tok[0]
                    if "s" in tok[1:]:
                        n, s = tok[1:].split("s")
                        runs.append((kind, int(n), int(s)))
                    else:
                        runs.append((kind, int(tok[1:]), 0))
            elif line.startswith("sink_len:"):
                sink_len = int(line.split(":")[1])
            elif line.startswith("class"):
                cur = CLASS_ID[line.split()[1]]
                masks[cur] = []
            else:
                masks[cur].append(line)
    pos, spans = 0, []
    for kind, n, s in runs:
        if kind == "I":
            spans.append((pos, pos + n, s))
        pos += n
    L = pos
    out = {}
    for c, rows in masks.items():
        assert len(rows) == L, (path, c)
        m = np.zeros((L, L), dtype=np.uint8)
        for i, r in enumerate(rows):
            assert len(r) == i + 1, (path, c, i)
            m[i, : i + 1] = [int(ch) for ch in r]
        out[c] = m
    return L, np.asarray(spans, dtype=np.int32).reshape(-1, 3), sink_len, out


def all_fixtures():
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    return sorted(glob.glob(os.path.join(here, "masks_*.txt")))


def load_full(path):
    """Fixtures with full-width rows, an `offsets:` line (sink offsets inside every image), a
    `mode:` line (bidir = non-causal attention inside an image) and an optional `window:` line."""
    runs, sink_len, offsets, mode, masks, cur, window = None, 0, [], "causal", {}, None, 0
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line.startswith("runs:"):
                runs = []
                for tok in line[5:].split():
                    n, _, s = tok[1:].partition("s")
                    runs.append((tok[0], int(n), int(s or 0)))
            elif line.startswith("offsets:"):
                offsets = [int(x) for x in line.split(":")[1].split()]
            elif line.startswith("sink_len:"):
                sink_len = int(line.split(":")[1])
            elif line.startswith("mode:"):
                mode = line.split(":")[1].strip()
            elif line.startswith("window:"):
                window = int(line.split(":")[1])
            elif line.startswith("class"):
                cur = CLASS_ID[line.split()[1]]
                masks[cur] = []
            else:
                masks[cur].append(line)
    pos, spans = 0, []
    for kind, n, s in runs:
        if kind == "I":
            spans.append((pos, pos + n, s))
        pos += n
    out = {}
    for c, rows in masks.items():
        assert len(rows) == pos and all(len(r) == pos for r in rows), (path, c)
        out[c] = np.array([[int(ch) for ch in r] for r in rows], dtype=np.uint8)
    return pos, np.asarray(spans, dtype=np.int32).reshape(-1, 3), sink_len, offsets, mode == "bidir", out, window


def full_fixtures():
    here = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")
    return sorted(glob.glob(os.path.join(here, "bidir_masks_*.txt")))
