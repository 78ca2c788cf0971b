"""MI355X-native Skip-FFN block (Skip-Vision, Section 4.2).

The GPU entry points live in `paper_2503_21817_amd.binding` (a ctypes layer
over the C-ABI library built from `csrc/`); it is imported lazily so that the
input generators and the cost model can be used on a machine with no GPU.
"""

__all__ = ["binding", "workloads", "flopmodel"]
