"""MI355X (gfx950) implementation of the ActionStudio fine-tuning step.

`binding` loads libactionstudio.so (built by `build.py`) and exposes the C
interface of include/actionstudio.h with the same names; it raises on import
when the library has not been built.
"""
