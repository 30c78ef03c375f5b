"""The five synthetic benchmark configurations: which schedule file, element type, size, value recipe and seed.

Plain data only.  "bytes_per_rank" is the whole rank buffer (G chunks), for both collectives.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, List, Optional


@dataclass(frozen=True)
class Workload:
    name: str
    schedule: str            # file under schedules/
    dtype: str               # i32 | f32 | f16
    dist: str                # inputs.generate distribution
    seed: int
    bytes_per_rank: int      # the whole rank buffer: every chunk position the layout gives a rank
    poison_non_owned: bool   # non-combining collectives: positions a rank holds nothing in at the start are undefined inputs
    options: Optional[Dict[str, int]] = None   # a launch shape found by `bench.py --workload W --sweep`, where one beats the plan's own choice (none does at present)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "f16" else 4


MiB = 1 << 20

WORKLOADS: Dict[str, Workload] = {
    # config 1: Allgather on the 4-ring, 1024 fp32 per chunk
    "cfg1": Workload("cfg1", "cfg1_allgather_ring4", "f32", "uniform", 1, 4 * 1024 * 4, True),
    # config 2: Allgather on the 8-node graph, 8 ranks x 64 MiB int32
    "cfg2": Workload("cfg2", "cfg2_allgather_hcm8", "i32", "u32", 2, 64 * MiB, True),
    # config 3 (headline): Allreduce fp32, 8 ranks x 256 MiB
    "cfg3": Workload("cfg3", "cfg3_allreduce_hcm8", "f32", "uniform", 3, 256 * MiB, False),
    # config 4: ring Allreduce fp16 (fp32 accumulation), 8 ranks x 512 MiB
    "cfg4": Workload("cfg4", "cfg4_allreduce_ring8", "f16", "normal", 4, 512 * MiB, False),
    "cfg4b": Workload("cfg4b", "cfg4b_allreduce_ring8_c2", "f16", "normal", 4, 512 * MiB, False),
    # beyond the five configurations: Alltoall, the paper's row (8,3,3) on its DGX-1 graph; 8 ranks, 8 MiB chunks
    # (a 64 MiB send buffer per rank) in a compact layout of 20 chunk positions per rank
    "alltoall": Workload("alltoall", "alltoall_dgx1", "f32", "uniform", 6, 20 * 8 * MiB, True),
    # and the other collectives of the paper's Table 2 on the same graph, 64 MiB rank buffers
    "broadcast": Workload("broadcast", "broadcast_dgx1", "f32", "uniform", 7, 64 * MiB, True),
    "reduce": Workload("reduce", "reduce_dgx1", "f32", "uniform", 8, 64 * MiB, False),
    "gather": Workload("gather", "gather_dgx1", "f32", "uniform", 9, 64 * MiB, True),
    "scatter": Workload("scatter", "scatter_dgx1", "f32", "uniform", 10, 64 * MiB, True),
    # and Reducescatter, the inverted Allgather (2,3,3) of the paper's Table 4, 16 chunks of 16 MiB per rank
    "reducescatter": Workload("reducescatter", "reducescatter_dgx1", "f32", "uniform", 11, 256 * MiB, False),
}


def sweep_sizes() -> List[int]:
    """Config 5: per-rank buffer 1 KiB .. 1 GiB in powers of 4."""
    return [1024 * 4 ** i for i in range(11)]


def sweep_workload(collective: str, bytes_per_rank: int, algorithm: str = "bandwidth") -> Workload:
    """Config 5 at one size.  algorithm: "bandwidth" = the greedy schedule with four chunks per node, (4,15,15),
    bandwidth-optimal on the torus; "latency" = the exact search's (1,4,4), as many steps as the diameter."""
    assert collective in ("allgather", "allreduce") and algorithm in ("bandwidth", "latency")
    suffix = "" if algorithm == "bandwidth" else "_latency"
    return Workload(f"cfg5_{collective}_{bytes_per_rank}{suffix}", f"cfg5_{collective}_torus4x4{suffix}", "f32", "uniform", 5,
                    bytes_per_rank, collective == "allgather")
