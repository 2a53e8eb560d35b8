"""MI355X-native stage-slicing dynamic program of Alpa's inter-operator pass (Sec. 5.2).

``binding`` is the thin ctypes layer over the C-ABI HIP library (``include/alpa_dp.h``);
``workloads`` makes seeded synthetic inputs; ``counts`` holds the work-unit bookkeeping.
Nothing here falls back to a CPU implementation: calling into ``binding`` without the
built HIP library raises.
"""
