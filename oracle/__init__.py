"""CPU oracle for shared-prefix decode attention and cache growth -- TEST INFRASTRUCTURE ONLY.

Plain, slow, fp64 numpy.  Only tests, the smoke check and the benchmark's
cpu_baseline leg may import this package; the product path (the HIP library and
its Python binding) never does, and this package imports nothing from it.

Parity pins (tests/test_oracle_*.py): brute-force dense attention in Python
loops, closed forms, placement/permutation invariance, split-and-merge
exactness, a library SDPA for the single-model case, the e4m3 format table, and
the Eq. 9 block-count / refcount invariants.  The cache-writing side (e4m3
encoder, ingest, append, table growth; tests/test_oracle_kv_update.py) is pinned
by the format table, an independently written quantiser, exact round trips,
error bounds, order-of-arrival identities between append and ingest, scalar
brute force and a hand-worked table.  The third sharing level (layout.build_layout_tree, a
context several prompts begin with; tests/test_oracle_tree.py) is pinned by a hand-worked table, the
block-count and refcount invariants, brute-force dense attention and bitwise identity with the
two-level oracle on the flattened batch.  Adoption of a cached context's blocks by a later layout (layout.build_layout(adopt=...);
tests/test_oracle_layout.py) is pinned by a hand-worked instance, its rules, and attention over the
continued context against the unpaged definition.  Staging of cold blocks (staging.py; tests/test_oracle_staging.py)
is pinned by a hand-worked park / resume sequence, the block-count identity, and the requirement that
a parked, overwritten and resumed batch reads back bit for bit.  No function here is unpinned.
"""
from . import attention, fp8, kv_update, layout, staging  # noqa: F401
