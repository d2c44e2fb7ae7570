"""The synthetic configurations the build is tested and timed on.

They stand in for the paper's Wan2.1 (80K tokens) and HunyuanVideo (127K
tokens) runs at 768x1280 (Sec. 5.1), whose models, prompts and searched masks
are not available: grids have the same token counts and tile shapes, and the
per-head window parameters are a seeded mix of the local / cross / global
spatial patterns and time-variant / time-invariant temporal patterns of
Sec. 3.2.

A head is a list of groups `(max_dt, (rh, rw), (rh, rw))`: tile-frame distance
bound and two window radii in tiles (negative = absent).

Pattern codes: `L r` one window (r, r); `C a` two windows (a, nW-1) and
(nH-1, a), i.e. full-length arms of thickness 2a+1; `G` one window covering
the whole tile grid.  A table entry `kind/F1/F2` means groups
[(F1, kind)] plus [(F2, L1)] when F2 > F1.
"""
from dataclasses import dataclass, field

ABSENT = (-1, -1)


def _ceil_div(a, b):
    return -(-a // b)


def windows_of(kind, nH, nW):
    """(window_a, window_b) of a pattern code on an nH x nW tile grid."""
    if kind == "G":
        return (nH - 1, nW - 1), ABSENT
    if kind[0] == "L":
        r = int(kind[1:])
        return (r, r), ABSENT
    if kind[0] == "C":
        a = int(kind[1:])
        return (a, nW - 1), (nH - 1, a)
    raise ValueError(kind)


def head_from_code(code, nH, nW):
    """`kind/F1/F2[=nnz]` -> (groups, expected nnz or None)."""
    nnz = None
    if "=" in code:
        code, nnz = code.split("=")
        nnz = int(nnz)
    kind, f1, f2 = code.split("/")
    f1, f2 = int(f1), int(f2)
    a, b = windows_of(kind, nH, nW)
    groups = [(f1, a, b)]
    if f2 > f1:
        groups.append((f2, (1, 1), ABSENT))
    return groups, nnz


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int                 # index into the benchmark's configs (1-based), seeds the values
    T: int
    H: int
    W: int
    tile: tuple              # (tt, th, tw)
    n_text: int
    num_heads: int
    head_dim: int
    dtype: str               # "f32" or "bf16"
    heads: tuple = field(repr=False)          # per head: list of groups
    expected_nnz: tuple = field(default=None, repr=False)   # per head, when tabulated
    batch: int = 1

    @property
    def seed(self):
        return 2508 * 10 + self.cfg

    @property
    def tiles(self):
        tt, th, tw = self.tile
        return _ceil_div(self.T, tt), _ceil_div(self.H, th), _ceil_div(self.W, tw)


# kind/F1/F2=nnz per head; nnz is the closed-form count of kept tile pairs for
# that head (text rows and columns included), tabulated independently of any code here.
_CFG3 = """
0:C0/4/4=152100   1:G/5/5=723600    2:C0/6/7=220444   3:G/7/7=932400    4:L1/1/1=27328    5:C0/7/9=255500
6:G/20/20=1587600 7:G/20/20=1587600 8:C1/4/4=365040   9:C1/5/7=460144   10:C1/5/6=447600  11:G/20/20=1587600
12:G/7/7=932400   13:C0/1/3=88052   14:L1/5/6=103488  15:L3/1/3=139292  16:C0/2/2=89100   17:G/20/20=1587600
18:C1/5/7=460144  19:L2/4/5=192800  20:L1/1/1=27328   21:C1/2/4=245200  22:C1/2/3=229968  23:L1/2/4=75712
24:L1/5/6=103488  25:L2/5/7=238240  26:C1/7/9=581840  27:C1/7/7=559440  28:L2/8/9=311712  29:C1/8/10=636208
30:G/20/20=1587600 31:C0/0/2=53844  32:C0/4/4=152100  33:C0/2/2=89100   34:G/20/20=1587600 35:L1/6/7=116032
36:G/0/0=75600    37:C1/4/5=379376  38:L3/3/4=250132  39:C1/4/4=365040
"""
_CFG4_S50 = """
0:C0/6/6=165184   1:G/7/7=720484    2:G/16/16=1044484 3:G/8/8=785284    4:L1/2/2=39476    5:C0/8/10=212824
6:G/16/16=1044484 7:G/16/16=1044484 8:C1/5/5=343204   9:G/6/8=665508    10:G/16/16=1044484 11:G/16/16=1044484
12:G/16/16=1044484 13:C0/1/3=74168  14:L1/6/7=93236   15:L3/1/3=115328  16:C0/3/3=100384  17:G/16/16=1044484
18:G/16/16=1044484 19:L2/6/7=202068 20:L1/2/2=39476   21:C1/3/5=257604  22:C1/2/3=187268  23:L1/3/5=74420
"""
_CFG4_S65 = """
0:C0/4/4=123784   1:G/5/5=569284    2:C0/5/6=155240   3:G/6/6=648484    4:L1/1/1=26036    5:C0/6/8=182208
6:G/16/16=1044484 7:G/16/16=1044484 8:C1/4/4=291364   9:C1/4/6=311972   10:C1/5/6=353060  11:G/16/16=1044484
12:G/6/6=648484   13:C0/1/3=74168   14:L1/4/5=74420   15:L3/1/3=115328  16:C0/2/2=75184   17:G/16/16=1044484
18:C1/5/7=362020  19:L2/4/5=155284  20:L1/1/1=26036   21:C1/2/4=198916  22:C1/1/2=123364  23:L1/2/4=63668
"""
_CFG4_S80 = """
0:C0/2/2=75184    1:G/3/3=389284    2:C0/3/4=112032   3:G/4/4=482884    4:L1/1/1=26036    5:C0/4/6=144392
6:G/4/6=503492    7:G/4/5=493636    8:C1/2/2=174724   9:C1/3/5=257604   10:C1/3/4=246852  11:G/0/2=93060
12:G/3/3=389284   13:C0/0/2=47160   14:L1/3/4=63668   15:L3/0/2=61440   16:C0/1/1=48184   17:G/16/16=1044484
18:C1/3/5=257604  19:L2/2/3=100052  20:L1/1/1=26036   21:C1/1/3=135908  22:C1/1/2=123364  23:L1/1/3=52020
"""
_CFG5 = """
0:C0/2/2=138600   1:G/3/3=763200    2:C0/3/4=215888   3:C1/4/4=578880   4:L1/1/1=42112    5:C0/4/6=288688
6:G/4/6=1012288   7:G/4/5=988992    8:C1/2/2=332640   9:C1/3/5=507200   10:C1/3/4=483008  11:C1/0/2=123776
12:C0/3/3=190800  13:L1/0/2=68992   14:L1/3/4=120064  15:L3/0/2=110336  16:C0/1/1=84600   17:C0/0/1=56576
18:C1/3/5=507200  19:L2/2/3=188608  20:L1/1/1=42112   21:C1/1/3=255904  22:C1/1/2=229920  23:L1/1/3=94976
"""


def _from_table(table, nH, nW):
    entries = {}
    for item in table.split():
        idx, code = item.split(":")
        entries[int(idx)] = head_from_code(code, nH, nW)
    heads = tuple(entries[i][0] for i in range(len(entries)))
    nnz = tuple(entries[i][1] for i in range(len(entries)))
    return heads, nnz


def _cfg1():
    nH, nW = 2, 2
    heads = ([(1, *windows_of("L1", nH, nW))], [(3, *windows_of("C0", nH, nW))])
    return Workload("cfg1", 1, 4, 8, 8, (1, 4, 4), 0, 2, 64, "f32", heads, (160, 192))


def _cfg2():
    nH, nW = 4, 4
    kinds = ("L1", "C0", "G")
    heads = tuple(
        [(0, *windows_of("G", nH, nW)), (2, *windows_of(kinds[h % 3], nH, nW)), (7, *windows_of("L1", nH, nW))]
        for h in range(12)
    )
    nnz = tuple((7648, 7960, 11704)[h % 3] for h in range(12))
    return Workload("cfg2", 2, 8, 32, 32, (1, 8, 8), 0, 12, 64, "bf16", heads, nnz)


def _cfg3():
    heads, nnz = _from_table(_CFG3, 6, 10)
    return Workload("cfg3", 3, 21, 45, 80, (1, 8, 8), 0, 40, 128, "bf16", heads, nnz)


def _cfg4(name, table):
    heads, nnz = _from_table(table, 6, 10)
    return Workload(name, 4, 33, 45, 80, (2, 8, 8), 256, 24, 128, "bf16", heads, nnz)


def _cfg5():
    heads, nnz = _from_table(_CFG5, 6, 10)
    return Workload("cfg5", 5, 64, 45, 80, (2, 8, 8), 0, 24, 128, "bf16", heads, nnz)


_BUILDERS = {
    "cfg1": _cfg1,
    "cfg2": _cfg2,
    "cfg3": _cfg3,
    "cfg4-S50": lambda: _cfg4("cfg4-S50", _CFG4_S50),
    "cfg4-S65": lambda: _cfg4("cfg4-S65", _CFG4_S65),
    "cfg4-S80": lambda: _cfg4("cfg4-S80", _CFG4_S80),
    "cfg5": _cfg5,
}
WORKLOAD_NAMES = tuple(_BUILDERS)


def get_workload(name):
    return _BUILDERS[name]()
