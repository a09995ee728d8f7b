"""MI355X-native NSA layer (3D-aware routing, block pooling, three-branch attention).

`paper_2604_05182_amd.inputs` holds the seeded workload generators and imports
nothing else; `paper_2604_05182_amd.binding` loads the HIP library (and raises if it
has not been built).  Nothing here falls back to a CPU implementation.
"""

__all__ = ["inputs", "binding", "build"]
