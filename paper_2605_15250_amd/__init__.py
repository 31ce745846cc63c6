"""GQLA decode attention for AMD MI355X (gfx950): thin Python binding over the C-ABI library libgqla.so.

Importing the package does not load the library; the first use of `paper_2605_15250_amd.binding` does,
and fails loudly if the library has not been built (`python -m paper_2605_15250_amd.build`)."""

__all__ = ["binding", "build"]
