"""Plain-data record layouts shared by every side (generator, oracle binding, HIP binding).

Only byte layouts live here: numpy structured dtypes that mirror the C structs of
``include/fdy.h`` field for field.  No arithmetic of the method is defined in this module.
"""
import numpy as np

ALLOC = np.dtype([("base", "<u8"), ("size", "<u8")])  # fdy_alloc, 16 B
NODE = np.dtype(
    [
        ("kernel_id", "<u8"),
        ("grid", "<u4", (3,)),
        ("block", "<u4", (3,)),
        ("blob_len", "<u4"),
        ("flags", "<u4"),
    ]
)  # fdy_node, 40 B
RELOC = np.dtype([("word", "<u4"), ("region", "<u4"), ("offset", "<u8")])  # fdy_reloc, 16 B
OVR32 = np.dtype([("byte_off", "<u4"), ("value", "<u4")])  # fdy_ovr32, 8 B
GRID_OVR = np.dtype([("node", "<u4"), ("grid", "<u4", (3,))])  # fdy_grid_ovr, 16 B
PATCH = np.dtype([("word", "<u4"), ("reserved", "<u4"), ("value", "<u8")])  # fdy_patch, 16 B

assert ALLOC.itemsize == 16 and NODE.itemsize == 40 and RELOC.itemsize == 16
assert OVR32.itemsize == 8 and GRID_OVR.itemsize == 16 and PATCH.itemsize == 16

# fingerprint field-mask bits (values of the FDY_FP_* macros)
FP_KERNEL_ID = 0x01
FP_GRID_X = 0x02
FP_GRID_Y = 0x04
FP_GRID_Z = 0x08
FP_BLOCK = 0x10
FP_BLOB_LEN = 0x20
FP_FLAGS = 0x40
FP_ALL = 0x7F

# device status bits (values of the FDY_ST_* macros)
ST_CAPACITY = 0x1
ST_BAD_INDEX = 0x2
ST_BAD_SIZE = 0x4
ST_SPIN = 0x8
ST_BAD_ORDER = 0x10
ST_BAD_PREPARED = 0x20
