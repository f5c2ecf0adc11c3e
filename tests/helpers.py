"""Small test-only helpers (fixture parsing); no method arithmetic."""
import os

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def load_hand_fixture(name="hand_2_2_6.txt"):
    sections, cur = {}, None
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            if line in ("mask", "columns", "values", "meta"):
                cur = line
                sections[cur] = []
                continue
            sections[cur].append([tok for tok in line.replace("|", " ").split()])
    mask = np.array([[int(t) for t in row] for row in sections["mask"]], dtype=np.uint8)
    R, K = mask.shape
    V, M = 2, 6
    G = K // M
    columns = np.array([[int(t) for t in row] for row in sections["columns"]], dtype=np.uint16).reshape(R // V, G, 4)
    values = np.array([[int(t, 16) for t in row] for row in sections["values"]], dtype=np.uint16).reshape(R, G, 2)
    meta = np.array([[int(t, 16) for t in row] for row in sections["meta"]], dtype=np.uint32)
    A_bits = (0x3C00 + 16 * np.arange(R)[:, None] + np.arange(K)[None, :]).astype(np.uint16)
    return dict(A_bits=A_bits, mask=mask, columns=columns, values=values, meta=meta, V=V, M=M, R=R, K=K)
