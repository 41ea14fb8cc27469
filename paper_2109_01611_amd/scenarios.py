"""Scheduler inputs: request scenarios, SLOs and seeded synthetic latency tables.

Like ``inputs`` this module serves both the CPU oracle and the library, so it
holds none of the scheduling arithmetic: it only lists the paper's scenario
tables and draws latency tables of the right shape.

* ``SIZES`` are the gpu-let sizes the paper profiles and splits a GPU into
  (Sec. 3.1, Fig. 3: 20-100%; splits 2:8, 4:6, 5:5, 6:4, 8:2), ``BATCHES`` the
  profiled batch sizes (1-32).
* ``PAPER_SLO_MS`` is Table 4; ``slo_from_table`` applies the rule behind that
  table (twice the solo latency of batch 32) to a measured or synthetic table.
* ``PAPER_SCENARIOS`` is Table 5; ``rate_grid`` enumerates the scenario grid
  of Sec. 3.1 (every model at one of four rates, all-zero excluded).
* ``synthetic_table`` draws an L(b, p) table with the structure of Fig. 3: a
  fixed launch cost plus work per image divided by the share of the GPU the
  batch can actually use, which saturates for small batches.
"""

import itertools

from . import inputs

SIZES = (20, 40, 50, 60, 80, 100)
BATCHES = (1, 2, 4, 8, 16, 32)

MODELS = ("le", "goo", "res", "ssd", "vgg")
PAPER_SLO_MS = {"goo": 44.0, "le": 5.0, "res": 95.0, "ssd": 136.0, "vgg": 130.0}

PAPER_SCENARIOS = {
    "equal": {"le": 50.0, "goo": 50.0, "res": 50.0, "ssd": 50.0, "vgg": 50.0},
    "long-only": {"le": 0.0, "goo": 0.0, "res": 100.0, "ssd": 100.0, "vgg": 100.0},
    "short-skew": {"le": 100.0, "goo": 100.0, "res": 100.0, "ssd": 50.0, "vgg": 50.0},
}

PAPER_RATE_LEVELS = (0.0, 200.0, 400.0, 600.0)


def rate_grid(n_models, levels=PAPER_RATE_LEVELS):
    """All assignments of one rate level per model except the all-zero one
    (4^5 - 1 = 1,023 for the paper's five models), in lexicographic order."""
    return [list(c) for c in itertools.product(levels, repeat=n_models) if any(v > 0 for v in c)]


def slo_from_table(table, sizes=SIZES, batches=BATCHES):
    """SLO in ms by the rule of Table 4: twice the latency of the largest
    profiled batch on the whole GPU."""
    return 2.0 * table[sizes.index(100)][len(batches) - 1]


def synthetic_table(seed, name, sizes=SIZES, batches=BATCHES):
    """Seeded L(b, p) in ms as nested lists [size][batch].

    L = t0 + w * b / min(p/100, min(1, b*u)): ``t0`` a fixed cost (0.05-0.5 ms),
    ``w`` the full-GPU time per image (0.02-2 ms, log-uniform), ``u`` the share
    of the GPU one image can fill (0.02-0.5, log-uniform), times a +-2% ripple
    per cell so that no two cells tie."""
    u = inputs.uniform(seed, "latency_table/" + name, 3 + len(sizes) * len(batches))
    t0 = 0.05 + 0.45 * u[0]
    w = 0.02 * (100.0 ** u[1])
    fill = 0.02 * (25.0 ** u[2])
    table, k = [], 3
    for p in sizes:
        row = []
        for b in batches:
            share = min(p / 100.0, min(1.0, b * fill))
            row.append(float((t0 + w * b / share) * (0.98 + 0.04 * u[k])))
            k += 1
        table.append(row)
    return table
