"""CPU oracle for the reshard data path.  TEST INFRASTRUCTURE ONLY.

Plain, slow, definitional implementations of what the GPU path must produce:
which elements of a holder's shard a reader needs, the byte stream they form
on the wire, where they land in the reader's shard, and the fp32 -> bf16
round-to-nearest-even narrowing.  Nothing here is tiled, fused or reordered,
and nothing is shared with the HIP library or its planner: only tests, the
smoke check and the benchmark's CPU-baseline leg may import this package.

The paper (TensorHub / Reference-Oriented Storage) states the mechanism only
in words - weights are resharded and converted to an inference-ready format
before transfer (Sec. 2.1, step 4); tensor data is copied slice by slice into
staging buffers (Sec. 4.3.2, "RDMA Copy"); tiny tensors are compacted into
contiguous buffers which the receiver unpacks into their slices (Sec. 4.3.2,
"Tiny-Tensor Optimization"); a reader consumes a prefix of the tensors
(Sec. 4.3.3).  It prints no layout math, no wire format and no worked example
for this path.  The conventions implemented here (standard tensor-parallel /
expert-parallel shard shapes, wire order, 16-byte tensor alignment, NaN rule)
are readings, each stated in the module that implements it; their pins are mathematical:
round trips, exactly-once coverage, byte conservation, brute force on tiny
shapes, agreement with numpy.split, exhaustive RNE checks.
"""
from . import rne, layouts, reshard, segments, checksum  # noqa: F401
