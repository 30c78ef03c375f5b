"""A second, independent executor of a schedule for the full-size GPU tests: plain PyTorch ops on the device.

It follows the same definition as the CPU oracle (sections 3.3 and 3.5 of the paper: per step, COPY sends replace
the destination's chunk, all REDUCE sends of a step into one (chunk, destination) are added left to right onto the
destination's own value in binary32 -- wrapping int32 for integers -- and binary16 is narrowed once per group), one
torch operation per operand, with no blocking or fusion.  It is NOT the oracle: the oracle stays the authority and
is run on element ranges of the same buffers in the same test.  What this adds is a comparison of EVERY byte of a
16 GiB working set in a fraction of a second, against kernels that are not this library's.
"""
import torch

TORCH_DTYPE = {"i32": torch.int32, "f32": torch.float32, "f16": torch.float16}


def execute(sf, dtype, epc, bufs):
    """Runs schedule file `sf` in place on the P device tensors `bufs` (each positions_per_rank * epc elements)."""
    K = sf.positions_per_rank
    views = [b.view(K, epc) for b in bufs]
    acc_dtype = torch.int32 if dtype == "i32" else torch.float32

    def at(c, n):
        return views[n][c if sf.slot is None else int(sf.slot[c, n])]

    steps = [[] for _ in sf.rounds]
    for c, n, m, s, op in sf.sends.tolist():
        steps[s].append((c, n, m, op))
    for sends in steps:
        taken = [False] * len(sends)
        for i, (c, n, m, op) in enumerate(sends):
            if taken[i]:
                continue
            if op == 0:
                at(c, m).copy_(at(c, n))
                continue
            acc = at(c, m).to(acc_dtype)
            for j in range(i, len(sends)):                 # the group: every REDUCE of this step into (c, m), in array order
                cj, nj, mj, opj = sends[j]
                if not taken[j] and opj == 1 and cj == c and mj == m:
                    taken[j] = True
                    acc = acc + at(c, nj).to(acc_dtype)
            at(c, m).copy_(acc.to(TORCH_DTYPE[dtype]))
