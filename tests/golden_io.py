"""Readers of the small text fixtures under tests/golden/ (values the paper prints)."""
import os

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def table4_params():
    """Table 4 (appendix): per ternary ResNet-18 layer the learned activation scale gamma,
    offset beta and the mean weight scale -> list of (layer name, gamma, beta, mean alpha)."""
    rows = []
    with open(os.path.join(GOLD, "table4_resnet18_params.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, g, b, a = line.split()
            rows.append((name, float(g), float(b), float(a)))
    return rows
