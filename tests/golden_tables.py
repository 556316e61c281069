"""Loads the paper's Table 2 fixture as a cost table (rows = n_q axis, cols = n axis)."""
import os


def load_table2():
    path = os.path.join(os.path.dirname(__file__), "golden", "table2_block_time_us.txt")
    len_grid, cols = [], None
    rows = []
    for line in open(path):
        if line.startswith("# n_q:"):
            cols = [int(x) for x in line.split(":")[1].split()]
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x) for x in line.split()]
        len_grid.append(v[0])
        rows.append(v[1:])
    # cost[ri][ni]: first index over the query-count axis
    cost = [[rows[ni][ri] for ni in range(len(len_grid))] for ri in range(len(cols))]
    return {"row_grid": cols, "len_grid": len_grid, "cost": cost}
