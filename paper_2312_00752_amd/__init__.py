"""MI355X-native selective scan (the selective SSM operator of arXiv 2312.00752).

``paper_2312_00752_amd.workloads`` draws the seeded synthetic inputs;
``paper_2312_00752_amd.binding`` is the thin ctypes layer over the C-ABI library built
from ``csrc/`` (imported on demand so that the input generators carry no GPU dependency).
"""
