"""MI355X-native Winograd-aware convolution forward path (F(m x m, 3 x 3), m in {2,4,6}).

The work is done by hand-written HIP kernels for gfx950 behind a C ABI
(``include/wino.h``, built into ``libwino.so``).  ``binding`` marshals arguments
to it; ``workloads`` draws the seeded synthetic inputs.  Nothing here computes on
the CPU: if the library is missing the binding raises.
"""

__all__ = ["binding", "workloads"]
