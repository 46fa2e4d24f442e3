"""libflashd for MI355X (gfx950): the FlashAttention forward pass in the
FLASH-D form (sigmoid-weighted blend, no softmax division, no running max).

`paper_2505_14201_amd.flashd` is the thin ctypes binding over the C-ABI shared
library; `paper_2505_14201_amd.synthetic` draws the seeded inputs.  Importing
the package itself touches neither, so the input generators stay usable on a
machine without the built library; calling into `flashd` without it raises.
"""

__all__ = ["flashd", "synthetic"]
