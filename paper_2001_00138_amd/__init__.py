"""MI355X-native pattern-sparse 3x3 convolution (PatDNN inference hot path).

The package holds:

* ``workloads``  - seeded synthetic layer generators (shapes of the paper's
  VGG-16 / ResNet-50 / MobileNet-V2 workloads, section 6.1).  Pure data, none
  of the method's arithmetic; serves both the HIP path and the test oracle.
* ``binding``    - ctypes marshalling over the C-ABI library ``libpatdnn.so``
  (declared in ``include/patdnn.h``).  Every step of the path runs in the HIP
  library; there is no CPU fallback.
* ``buildlib``   - compiles ``csrc/`` for gfx950 with hipcc.
* ``profile_summary`` - turns rocprofv3 CSVs into the short summaries kept in
  ``profiles/``.

Importing the package does not load the shared library; ``binding`` does so on
first use and raises if it is missing.
"""

__all__ = ["workloads", "binding", "buildlib", "profile_summary"]
