"""Seeded synthetic scheduling problems (operator placements) used by tests and the benchmark.

This module only *describes* problems -- blocks, the simulated devices they occupy,
dependencies, integer times and memory deltas, cap, repetend size, candidate space, seed.
It holds none of the evaluator's arithmetic and is the one module that both the HIP
library's callers and the CPU oracle's callers import.

Block types are numbered along the micro-batch's dependency chain:
F_0 .. F_{S-1}, B_{S-1} .. B_0 (Sec. III-A: K blocks per micro-batch, forward blocks create
memory, backward blocks release it).
"""

_MASK64 = (1 << 64) - 1


class _Stream:
    """SplitMix64 sequence; uniform integers by modulo (ranges here are tiny)."""

    def __init__(self, seed):
        self.x = seed & _MASK64

    def next(self):
        self.x = (self.x + 0x9E3779B97F4A7C15) & _MASK64
        z = self.x
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
        return z ^ (z >> 31)

    def randint(self, lo, hi):
        return lo + self.next() % (hi - lo + 1)


def pipeline_problem(stage_dev, tf, tb, num_devices, nr, mem_cap, space, seed=0, lead_step_q16=0,
                     fixed_leads=None, name="pipeline"):
    """Stages placed on single devices; chain F_0->..->F_{S-1}->B_{S-1}->..->B_0; m = +1 / -1."""
    S = len(stage_dev)
    t = list(tf) + list(reversed(tb))
    m = [1] * S + [-1] * S
    dev = list(stage_dev) + list(reversed(stage_dev))
    return {
        "name": name, "D": num_devices, "K": 2 * S, "NR": nr, "M": mem_cap,
        "t": t, "m": m, "dev_mask": [1 << d for d in dev],
        "deps": [(i, i + 1) for i in range(2 * S - 1)],
        "space": space, "seed": seed, "lead_step_q16": lead_step_q16, "fixed_leads": fixed_leads,
    }


def linear_placement(p):
    return list(range(p))


def folded_placement(num_devices):
    """'V' of 2*D stages folded over D devices: stage s on device s, then back down."""
    return list(range(num_devices)) + list(reversed(range(num_devices)))


def config1():
    """2 devices, 1 stage each, tf=1 tb=2, cap 2, N_R=2; every per-device ordering (576)."""
    return pipeline_problem(linear_placement(2), [1, 1], [2, 2], 2, 2, 2, "factorial", name="cfg1-2dev-exhaustive")


def config2():
    """4 devices, linear 4 stages, tf=1 tb=2, cap 4, N_R=4; all canonical candidates."""
    return pipeline_problem(linear_placement(4), [1] * 4, [2] * 4, 4, 4, 4, "canonical", name="cfg2-4dev-linear")


def config3(space="sampled_repair", seed=0x3C0FFEE3):
    """8 stages folded on 4 devices, tf in {1..3} seeded, tb = 2 tf, cap 6, N_R=4; 2^24 samples."""
    rng = _Stream(seed)
    tf = [rng.randint(1, 3) for _ in range(8)]
    tb = [2 * x for x in tf]
    prob = pipeline_problem(folded_placement(4), tf, tb, 4, 4, 6, space, seed=seed, lead_step_q16=32768,
                            name="cfg3-4dev-vshape")
    prob["n_candidates"] = 1 << 24
    return prob


def config4(space="sampled_repair", seed=0x4C0FFEE4):
    """4 devices; a tensor-parallel embedding block on all of them (tf=2, tb=4, m=+2/-2) around
    4 pipelined stages (tf in {1..3} seeded, tb = 2 tf, m=+1/-1); cap 6, N_R=4; 2^26 samples.
    Chain: E_F -> S0_F..S3_F -> S3_B..S0_B -> E_B (tied embedding/head as one block type)."""
    rng = _Stream(seed)
    tf = [rng.randint(1, 3) for _ in range(4)]
    t = [2] + tf + [2 * x for x in reversed(tf)] + [4]
    m = [2] + [1] * 4 + [-1] * 4 + [-2]
    masks = [0xF] + [1 << s for s in range(4)] + [1 << s for s in reversed(range(4))] + [0xF]
    return {
        "name": "cfg4-4dev-interlaced", "D": 4, "K": 10, "NR": 4, "M": 6, "t": t, "m": m, "dev_mask": masks,
        "deps": [(i, i + 1) for i in range(9)], "space": space, "seed": seed, "lead_step_q16": 32768,
        "fixed_leads": None, "n_candidates": 1 << 26,
    }


def config5(space="sampled_repair", seed=0x5C0FFEE5):
    """16 stages folded on 8 devices, tf in {1..4}, tb in {tf..3 tf} seeded, cap 10, N_R=8;
    2^28 samples, completion to 64 micro-batches."""
    rng = _Stream(seed)
    tf = [rng.randint(1, 4) for _ in range(16)]
    tb = [rng.randint(x, 3 * x) for x in tf]
    prob = pipeline_problem(folded_placement(8), tf, tb, 8, 8, 10, space, seed=seed, lead_step_q16=4096,
                            name="cfg5-8dev-vshape")
    prob["n_candidates"] = 1 << 28
    prob["num_microbatches"] = 64
    return prob


def xshape_problem(p, tf, tb, nr, cap, space="sampled_repair", seed=0x7C0FFEE7, lead_step_q16=20000):
    """Bidirectional pipelines over p devices (the X-shape placement of Chimera, Sec. VI-A): every micro-batch makes one
    pass down the devices and one pass up, two independent chains of 2p blocks, four block types per device."""
    t = [tf] * p + [tb] * p + [tf] * p + [tb] * p
    m = [1] * p + [-1] * p + [1] * p + [-1] * p
    down, up = list(range(p)), list(reversed(range(p)))
    masks = [1 << s for s in down + up + up + down]
    deps = [(i, i + 1) for i in range(2 * p - 1)] + [(2 * p + i, 2 * p + i + 1) for i in range(2 * p - 1)]
    return {"name": "xshape-%ddev" % p, "D": p, "K": 4 * p, "NR": nr, "M": cap, "t": t, "m": m, "dev_mask": masks,
            "deps": deps, "space": space, "seed": seed, "lead_step_q16": lead_step_q16, "fixed_leads": None}


def nnshape_problem(p, nr, cap, tf=1, tb=2, space="sampled_repair", seed=0x11C0FFEE, lead_step_q16=20000):
    """Two forward passes over the p devices, then two backward passes (the NN-shape of Sec. VI-A: an encoder pipeline
    followed by a decoder pipeline on the same devices): 2 p stages, four block types per device, one chain."""
    return pipeline_problem(list(range(p)) + list(range(p)), [tf] * (2 * p), [tb] * (2 * p), p, nr, cap, space, seed=seed,
                            lead_step_q16=lead_step_q16, name="nnshape-%d" % p)


def kshape_problem(nr, cap, tf=(2, 1, 3), tb=(4, 2, 6), space="sampled_repair", seed=0x8C0FFEE8, lead_step_q16=20000):
    """Two branches that join (the K-shape of Sec. VI-A: two encoders feeding a joint stage): A on device 0 and B on
    device 1 run side by side, J on device 2 needs both; the backward pass fans out again.  Types: A_F, B_F, J_F,
    J_B, A_B, B_B; dependencies A_F -> J_F, B_F -> J_F, J_F -> J_B, J_B -> A_B, J_B -> B_B."""
    t = [tf[0], tf[1], tf[2], tb[2], tb[0], tb[1]]
    return {"name": "kshape-3dev", "D": 3, "K": 6, "NR": nr, "M": cap, "t": t, "m": [1, 1, 1, -1, -1, -1],
            "dev_mask": [1, 2, 4, 4, 1, 2], "deps": [(0, 2), (1, 2), (2, 3), (3, 4), (3, 5)],
            "space": space, "seed": seed, "lead_step_q16": lead_step_q16, "fixed_leads": None}


def diamond_problem(nr, cap, space="sampled_repair", seed=0x9C0FFEE9, lead_step_q16=24000):
    """A stage that feeds two parallel stages which join again, forward and backward, on 4 devices (fan-out and
    fan-in on both passes): S_F(0) -> L_F(1), R_F(2) -> T_F(3) -> T_B(3) -> L_B(1), R_B(2) -> S_B(0)."""
    t = [1, 2, 3, 1, 2, 4, 5, 2]
    return {"name": "diamond-4dev", "D": 4, "K": 8, "NR": nr, "M": cap, "t": t, "m": [1, 1, 1, 1, -1, -1, -1, -1],
            "dev_mask": [1, 2, 4, 8, 8, 2, 4, 1],
            "deps": [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (4, 5), (4, 6), (5, 7), (6, 7)],
            "space": space, "seed": seed, "lead_step_q16": lead_step_q16, "fixed_leads": None}


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}
