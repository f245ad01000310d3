"""Helpers that drive the C-ABI library from a workloads TaskSet / a golden scenario."""
import numpy as np

import paper_2504_08795_amd as D
import workloads as wl


class Session:
    """daris_init ... daris_shutdown as a context manager."""

    def __init__(self, flags, device=0, seed=0):
        self.flags, self.device, self.seed = flags, device, seed

    def __enter__(self):
        D.daris_init(self.device, self.seed, self.flags)
        return self

    def __exit__(self, *exc):
        D.daris_shutdown()
        return False


def register_plain_tasks(n_streams, tasks):
    """Host-logic runs: one partition per entry of n_streams, tasks as 1-layer dummy DNNs cut by afet length.
    tasks: list of dict(period, deadline, prio, afet=[...])."""
    for ns in n_streams:
        p = D.daris_create_partition(8)
        if ns != 1:
            D.daris_partition_set_streams(p, ns)
    N = wl.nets
    for t in tasks:
        k = len(t["afet"])
        layers = [N.Layer(op=N.OP_CONV, c_in=4, c_out=4, k=1, in_from=i - 1) for i in range(k)]
        dnn, keep = D.make_dnn(layers, None, (4, 2, 2), "fp32")
        h = D.daris_register_task(dnn, t["period"], t["deadline"], t["prio"])
        D.daris_split_stages(h, k)
        for j, a in enumerate(t["afet"]):
            D.daris_set_afet(h, j, a)


def load_et(et_table, n_parts):
    for i, per_stage in enumerate(et_table):
        for j, per_part in enumerate(per_stage):
            for k in range(n_parts):
                v = np.asarray(per_part[k], np.int64)
                D.daris_set_virtual_time(i, j, k, 0, len(v), v)


def run_commands(cmds, d_in=None, d_out=None):
    """cmds: ("release", t, task) / ("migrate", t, task, part), time-sorted.  Returns release decisions."""
    dec = []
    for c in cmds:
        if c[0] == "release":
            dec.append(D.daris_release_job(c[2], None if d_in is None else d_in[c[2]], None if d_out is None else d_out[c[2]], c[1]))
        else:
            D.daris_migrate(c[2], c[3])
    D.daris_run_until_idle()
    return dec
