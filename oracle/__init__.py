"""CPU oracle for tree verification (test infrastructure, not a product path).

Plain, slow, fp64 NumPy restatements of what the verification step of the
paper computes (Section 2.1 steps 2-3; the tree attention mask of Section
3.1.2 / Fig. "tree attention mask"), of the commit of the accepted path to
the KV cache that follows it, and of the draft head step and the growth of the draft tree that precede it
(Section 3.1.2 Eq. 2-5, Section 3.2 Eq. 6-8).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; it shares no code with
the HIP library and never calls it.
"""
from .tree_attention import ancestor_sets, tree_verify_attention  # noqa: F401
from .accept_path import accept_path, AcceptResult  # noqa: F401
from .commit_path import commit_path, committed_rows  # noqa: F401
from .paged_kv import gather_pages, scatter_rows  # noqa: F401
from . import draft_head  # noqa: F401
from . import draft_tree  # noqa: F401
