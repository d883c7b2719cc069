"""libmpq for MI355X: the data-parallel hot path of sensitivity-guided mixed-precision PTQ.

``paper_2302_01382_amd.mpq``        ctypes binding of the C ABI in ``include/mpq.h``
``paper_2302_01382_amd.workloads``  seeded synthetic inputs of the benchmark configurations
``paper_2302_01382_amd.build``      hipcc build of ``libmpq.so`` (in-tree)
"""
