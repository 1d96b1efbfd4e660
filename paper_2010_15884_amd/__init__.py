"""sysconv for AMD MI355X: 1-D / 2-D fp32 valid convolution as software systolic
arrays inside a wavefront (arXiv 2010.15884), behind the C ABI of include/sysconv.h.

``binding``        ctypes wrappers with the C entry points' names
``workloads``      seeded synthetic inputs of the benchmark workloads
``schedule_model`` the paper's space-time transforms and analytical model
``build``          compiles libsysconv.so for gfx950
"""
__all__ = ["binding", "workloads", "schedule_model", "build"]
