"""Shared test helpers: golden-fixture parsing and error metrics.  No method arithmetic."""
from __future__ import annotations

import json
import math
import os
from fractions import Fraction

import numpy as np

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def parse_scalar(tok: str) -> float:
    """'3', '-1/7', 'ln(2)', '-ln(2)' -> float."""
    tok = tok.strip()
    sign = 1.0
    if tok.startswith("-"):
        sign, tok = -1.0, tok[1:]
    if tok.startswith("ln(") and tok.endswith(")"):
        return sign * math.log(float(Fraction(tok[3:-1])))
    return sign * float(Fraction(tok))


def parse_matrix(rows) -> np.ndarray:
    return np.array([[parse_scalar(t) for t in row] for row in rows], dtype=np.float64)


def load_golden(name: str) -> dict:
    with open(os.path.join(GOLDEN, name), "r", encoding="utf-8") as f:
        return json.load(f)


def max_abs(a, b) -> float:
    a = np.asarray(a, np.float64); b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b))) if a.size else 0.0


def row_rel_l2(test, ref) -> np.ndarray:
    """Per-row ||test - ref||_2 / ||ref||_2 over the last axis."""
    test = np.asarray(test, np.float64); ref = np.asarray(ref, np.float64)
    num = np.sqrt(((test - ref) ** 2).sum(-1))
    den = np.sqrt((ref ** 2).sum(-1))
    return num / np.maximum(den, 1e-300)
