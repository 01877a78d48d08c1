"""Pipelined Demand Layering for MI355X (gfx950).

The product is the C-ABI library declared in ``include/demand_layering.h``;
``paper_2605_11678_amd.binding`` is its thin ctypes binding.  Importing the
package itself loads nothing native.
"""

__all__ = ["binding", "configs", "synth", "build"]
