"""The five workloads (and nine more shapes): cluster shapes of the paper's tables with seeded Gaussian gradients.

scheme/a/b follow the library's byz_build_assignment arguments: MOLS (l, r) or
Ramanujan (s, m).  `cmax` is the value the paper's Tables 3, 4, 6 print for that (graph, q) where one does.
"""
from collections import namedtuple

Config = namedtuple("Config", "name scheme a b K f l r q cmax d attack steps seed")

MOLS, RAMANUJAN = 0, 1

CONFIGS = [
    # MOLS l=5, r=3, reversed gradient x(-100), d = 2^20, q = 3
    Config("cfg1_mols5x3_d1M_reversed", MOLS, 5, 3, 15, 25, 5, 3, 3, 3, 1 << 20,
           {"kind": "reversed", "c": 100.0}, 1, 20101004 + 0),
    # ResNet-18-sized d, MOLS l=5, r=3, ALIE z=1.0, q = 4   (the headline workload)
    Config("cfg2_mols5x3_resnet18_alie", MOLS, 5, 3, 15, 25, 5, 3, 4, 5, 11173962,
           {"kind": "alie", "z": 1.0}, 1, 20101004 + 1),
    # MOLS l=7, r=3, reversed gradient, q = 5
    Config("cfg3_mols7x3_resnet18_reversed", MOLS, 7, 3, 21, 49, 7, 3, 5, 8, 11173962,
           {"kind": "reversed", "c": 100.0}, 1, 20101004 + 2),
    # K=25, f=25, r=l=5: the paper's Ramanujan Case 2 cluster (m=s=5), mixed ALIE / constant,
    # per-file gradient scale U(0.5, 2), q = 6
    Config("cfg4_ram5x5_resnet18_mixed", RAMANUJAN, 5, 5, 25, 25, 5, 5, 6, 4, 11173962,
           {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}, 1, 20101004 + 3),
    # ResNet-50-sized d, MOLS l=7, r=3, ALIE z=1.5, q = 6, 20 steps of fresh gradients
    Config("cfg5_mols7x3_resnet50_alie_20steps", MOLS, 7, 3, 21, 49, 7, 3, 6, 12, 25557032,
           {"kind": "alie", "z": 1.5}, 20, 20101004 + 4),
    # beyond the five: the paper's Table 5 cluster, MOLS l=7, r=5 (245 rows), mixed attack, q = 6
    Config("cfg6_mols7x5_resnet18_mixed", MOLS, 7, 5, 35, 49, 7, 5, 6, 4, 11173962,
           {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}, 1, 20101004 + 35),
    # Ramanujan Case 2 with m > s (Sec. 4.2.1): m=7, s=5, (K,f,l,r) = (25,35,7,5), 175 rows,
    # reversed gradient, q = 6; c_max = 6 is the exhaustive search's value (no table prints it)
    Config("cfg7_ram5x7_resnet18_reversed", RAMANUJAN, 5, 7, 25, 35, 7, 5, 6, 6, 11173962,
           {"kind": "reversed", "c": 100.0}, 1, 20101004 + 57),
    # MOLS over F_9 (prime-power l, Sec. 4.1.1): (K,f,l,r) = (27,81,9,3), 243 rows, ALIE, q = 5;
    # c_max = 8 from the exhaustive search.  f > 64: single pass with two words per thread
    Config("cfg8_mols9x3_resnet18_alie", MOLS, 9, 3, 27, 81, 9, 3, 5, 8, 11173962,
           {"kind": "alie", "z": 1.0}, 1, 20101004 + 93),
    # Ramanujan Case 2 (Eq. 6) with r = 7 and with r = 5 at f > 64: (K,f,l,r) = (49,49,7,7),
    # (49,63,9,7), (25,65,13,5); 343, 441 and 325 rows; q = 5, c_max from the exhaustive search
    Config("cfg9_ram7x7_resnet18_mixed", RAMANUJAN, 7, 7, 49, 49, 7, 7, 5, 1, 11173962,
           {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}, 1, 20101004 + 77),
    Config("cfg10_ram7x9_resnet18_mixed", RAMANUJAN, 7, 9, 49, 63, 9, 7, 5, 2, 11173962,
           {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}, 1, 20101004 + 79),
    Config("cfg11_ram5x13_resnet18_mixed", RAMANUJAN, 5, 13, 25, 65, 13, 5, 5, 6, 11173962,
           {"kind": "mixed", "z": 1.0, "value": 1e3, "file_scales": True}, 1, 20101004 + 63),
    # MOLS over F_11 and F_13: (K,f,l,r) = (33,121,11,3) and (39,169,13,3), 363 and 507 rows,
    # ALIE, q = 4; c_max = 5 from the exhaustive search
    Config("cfg12_mols11x3_resnet18_alie", MOLS, 11, 3, 33, 121, 11, 3, 4, 5, 11173962,
           {"kind": "alie", "z": 1.0}, 1, 20101004 + 113),
    Config("cfg13_mols13x3_resnet18_alie", MOLS, 13, 3, 39, 169, 13, 3, 4, 5, 11173962,
           {"kind": "alie", "z": 1.0}, 1, 20101004 + 133),
    # the widest file count the library takes: Ramanujan Case 2 with s = 3, m = 85,
    # (K,f,l,r) = (9,255,85,3), 765 rows (34 GB); q = 2, c_max = 29 from the exhaustive search.
    # No single pass at this width: vote kernel, then the median over 255 winners
    Config("cfg14_ram3x85_resnet18_alie", RAMANUJAN, 3, 85, 9, 255, 85, 3, 2, 29, 11173962,
           {"kind": "alie", "z": 1.0}, 1, 20101004 + 385),
]
