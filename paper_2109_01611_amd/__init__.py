"""MI355X-native hot path behind gpu-lets (arXiv 2109.01611).

A gpu-let (paper Sec. 2.3) is a spatial partition holding p% of one GPU's
compute; here it is a CU-masked HIP stream.  The package holds

* ``inputs``    seeded synthetic tensors (no arithmetic of the method),
* ``workloads`` layer tables of the CNN shapes the paper serves (Table 4),
* ``gpulet``    the thin ctypes binding over the C-ABI library ``libgpulet.so``
                (conv / pool / FC kernels, partition manager, model runner,
                latency profiler),
* ``profiler``  the L(b, p) latency-table writer (paper Sec. 4.1, Table 2).

Importing the package loads nothing native; ``paper_2109_01611_amd.gpulet``
loads the shared library and raises if it has not been built.
"""

__all__ = ["inputs", "workloads", "gpulet", "profiler"]
