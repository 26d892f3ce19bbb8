"""CPU oracle for the OWQ mixed-precision linear layer.

TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library and
its Python binding) imports, links or runs this package; only the tests, the
smoke check and the bench's CPU-baseline leg do.  It is a plain, slow fp64
statement of what the layer computes and of the packed storage format, written
independently of the GPU code: the two share no code, tables or constants.

Pins (see tests marked "not gpu"):
  owq_linear_ref   k = 0 against an independently coded LUT + einsum route;
                   all-columns-weak against the plain fp16 matrix product;
                   hand-enumerated tiny layers; moving a column from the dense
                   to the weak set when its dequantised value is exact in fp16;
                   the pure-Python triple loop in `owq_linear_loops`.
  owq_linear_multi_ref
                   all tokens on one task against owq_linear_ref; the difference between two
                   task assignments against a plain matrix product with the difference of
                   the weak columns; nested Python loops on a tiny layer.
  pack / unpack    bit-exact round trip, byte count, a bit-by-bit scalar
                   address function written separately from the vectorised
                   packer, walking-ones patterns.
  bookkeeping      the closed forms and spot values of the paper's appendix D
                   and the memory row of the effective-bit sweep table.
  search_config    (configuration search of s and z) weights exactly on a quantiser grid with
                   and without an outlier that only a narrowed range absorbs, mirrored; weak
                   columns that must not move anything; reported error against the pinned
                   dequantiser; nested Python loops over the grid.  The grid itself is a
                   reading (the paper leaves it open): see oracle/search.py.
  owq_backward_ref (derivatives for weak-column tuning) the adjoint identities against the pinned
                   forward oracle, unit-vector responses entry by entry, central differences
                   of the forward loops, all columns weak, nested loops.
  Numerics of y on the paper's real checkpoints: parity unpinned (the paper
  prints no output values and ships no weights).
"""
