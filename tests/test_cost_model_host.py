"""The layout selection's cost arithmetic (Sec. "Data Layout Selection"), on made-up counts and costs: no GPU."""
from paper_1810_00845_amd import nets


def table(limbs, poly=None):
    costs = {op: 0.0 for op in nets.COST_OPS}
    costs.update(rot_left=100.0, add=1.0, limbs=limbs)
    if poly is not None:
        costs["poly"] = {op: (costs[op], 0.0, 0.0) for op in nets.COST_OPS}
        costs["poly"].update(poly)
    return costs


def counts_of(ops):
    """ops: [(operation, limbs)], one entry per occurrence."""
    c = {op: 0 for op in nets.COST_OPS}
    c["limb_sum"] = {op: 0 for op in nets.COST_OPS}
    c["limb_sq_sum"] = {op: 0 for op in nets.COST_OPS}
    for op, l in ops:
        c[op] += 1
        c["limb_sum"][op] += l
        c["limb_sq_sum"][op] += l * l
    return c


def test_flat_table_is_count_times_cost():
    c = counts_of([("rot_left", 8), ("rot_left", 4), ("add", 8)])
    assert nets.estimate_cost(c, table(8)) == 201.0


def test_level_aware_table_charges_each_occurrence_at_its_level():
    # a rotation costs 4 + 4 l + l^2: 100 at 8 limbs, 36 at 4, 16 at 2
    c = counts_of([("rot_left", 8), ("rot_left", 4), ("rot_left", 2), ("add", 8), ("add", 2)])
    costs = table(8, {"rot_left": (4.0, 4.0, 1.0)})
    assert nets.estimate_cost(c, costs) == 100.0 + 36.0 + 16.0 + 2.0
    assert nets.estimate_cost(c, costs, level_aware=False) == 302.0
    # every operation at the table's own level: the two figures agree
    top = counts_of([("rot_left", 8)] * 3)
    assert nets.estimate_cost(top, costs) == nets.estimate_cost(top, costs, level_aware=False) == 300.0
