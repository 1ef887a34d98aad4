"""MI355X (gfx950) native binary-network forward path after Espresso (arXiv 1705.07175).

``binding``  -- thin ctypes binding of the C ABI in ``include/espresso_hip.h``
``nets``     -- host drivers chaining the calls into the paper's MLP and CNN
``synth``    -- seeded synthetic inputs (no arithmetic of the method)
``build``    -- in-tree hipcc build of ``libespresso_hip.so``

The shared library is loaded on first use; there is no CPU fallback.
"""

__all__ = ["binding", "nets", "synth", "build"]
