"""Multi-world tensor data plane for one MI355X (arXiv 2407.08980's hot path).

The work is done by libmw.so (HIP kernels + host runtime, see include/mw.h);
`binding` exposes its C ABI one to one.  Importing this package loads nothing;
the library is opened by the first call into `binding`.
"""

__all__ = ["binding", "build"]
