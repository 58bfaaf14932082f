"""SSD-SGD parameter-update pipeline for MI355X (gfx950).

The work is done by the HIP library built from csrc/; `binding` is the thin
ctypes layer over its C ABI.  Nothing here falls back to a CPU path: using the
binding without the built library raises.
"""
