"""LUT-NN table-lookup linear operator (arXiv 2302.03213) for AMD MI355X: Python binding of
liblutnn.so.  Importing this package loads the HIP library and fails if it is absent."""
from .binding import (LIB, TABLE_F32, TABLE_I4, TABLE_I8, VARIANT_AUTO, VARIANT_FUSED, VARIANT_LDS,  # noqa: F401
                      VARIANT_MFMA, VARIANT_SMFMAC, LutLayer, LutTree, LutnnError, auto_variant, build_table,
                      conv2d, conv2d_rows, conv2d_tree, conv_geom, encode, encode_conv2d, encode_tree,
                      encode_tree_conv2d, encode_tree16, linear, linear_auto_variant, linear_tree16, lookup16,
                      linear_tree, lookup, set_tunable, softpq_backward, softpq_backward_static,
                      softpq_workspace_bytes, tunables, probe_smfmac_stream,
                      packed_bytes, table_bytes, version)
from . import cost  # noqa: F401
