"""MI355X-native HGRN2 recurrence (paper Section 3.2, Eq. 3): chunkwise forward/backward and the
single-token decode step as hand-written gfx950 kernels behind a C-ABI library.

The binding (and with it the native library) is loaded on first use, so that importing the
package -- e.g. for the seeded input generators in ``synth`` -- works on a machine without a GPU.
"""

__all__ = ["synth", "binding", "build"]
