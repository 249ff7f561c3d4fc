"""MI355X-native Encode stage (ViT forward, V_m = E(I_m); paper section 3.1, Eq. 1).

Sub-modules:
  workloads -- seeded synthetic inputs/weights for the five configurations (no arithmetic
               of the method itself; shared by the tests, the bench and the CPU oracle's
               callers)
  binding   -- ctypes binding of the C-ABI library ``libepd_encode.so`` (imports torch and
               loads the HIP library; import it explicitly)
  build     -- hipcc build of the library for gfx950

Nothing is imported eagerly so that ``workloads`` stays usable without the HIP library.
"""

__all__ = ["workloads", "binding", "build"]
