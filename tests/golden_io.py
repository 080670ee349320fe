"""Readers for the small text fixtures under tests/golden/ (values printed in the paper)."""
import os

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as fh:
        for line in fh:
            line = line.strip()
            if line and not line.startswith("#"):
                yield line


def table1_squares():
    squares, cur = {}, None
    for line in _lines("table1_mols_degree5.txt"):
        if line.startswith("L"):
            cur = int(line[1:])
            squares[cur] = []
        else:
            squares[cur].append([int(x) for x in line.split()])
    return squares


def table2_allocation():
    alloc = {}
    for line in _lines("table2_allocation_l5_r3.txt"):
        w, files = line.split(":")
        alloc[int(w)] = [int(x) for x in files.split()]
    return alloc


def distortion_tables():
    """{name: (scheme, a, b, [(q, cmax, eps_byz, eps_base, eps_frc, gamma), ...])}"""
    tables, cur = {}, None
    for line in _lines("distortion_tables.txt"):
        tok = line.split()
        if tok[0].startswith("table"):
            cur = tok[0]
            tables[cur] = (tok[1], int(tok[2]), int(tok[3]), [])
        else:
            tables[cur][3].append((int(tok[0]), int(tok[1]), float(tok[2]), float(tok[3]),
                                   float(tok[4]), float(tok[5])))
    return tables
