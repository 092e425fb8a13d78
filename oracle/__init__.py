"""Float64 CPU oracle for the selective-recompute prefill path (TEST INFRASTRUCTURE).

A plain, slow and deliberately unoptimised statement of what the path computes,
written from the paper's description of the linker and of selective attention
(Sec. 3.1, Sec. 4.1-4.2, Fig. 7, App. A) and from the position rule of the build
target (cached keys are rotated by the RoPE angle of their chunk's global offset).

It exists only to check the HIP library.  Nothing in the product path may import
it: only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg do.
It shares no code with the HIP path and never receives values from it.

Pin status of every function (see tests/test_oracle_*.py):
  plan.build_plan        pinned: hand-derived layout of the tiny config, closed-form
                         counts, brute-force set construction on random layouts
  rope.rotate            pinned: complex-multiplication form of RoPE, group laws
  link.link_kv           pinned: consistent-cache case reproduces full prefill
  link.position_fresh    pinned: row-by-row complex form of RoPE at per-request position
                         ids, full prefill reproduced from unpositioned fresh rows,
                         logits depend on the signed distance only
  link.link_kv_unshifted / attend.attend_unshifted   pinned: <Rot(-D) q, k> = <q, Rot(D) k> per
                         chunk instance (also against the complex form), and the pair gives
                         the outputs of link_kv + attend on random layouts, both pairings,
                         rotated and unrotated fresh rows
  attend.attend          pinned: loop transcription of App. A, library SDPA in the
                         recompute-all case, closed forms (zero queries, one-hot V)
  decode.decode_attend   pinned: the last row of causal prefill over context + new token
                         (library SDPA), the last row of attend when the request ends
                         in a text token, closed forms
  select.k_distance      pinned: loop transcription, closed forms (identical caches, a
                         constant offset), metric laws
  select.top_tokens / top_counts   pinned: hand-ranked example with ties, counts add up
  store.checksum / write_chunk_file / read_chunk_file   (this build's own encoding) pinned:
                         unbounded-integer evaluation, every single-byte change of a small
                         buffer and file is seen, hand-decoded header
  store.ChunkStore       pinned: hand-run sequence of put / move / expire / lookup
  pipeline.plan_with_lookup / prefill_layers   pinned: a missing or failed cache gives the
                         plan of a text span of the same length, all caches missing is
                         library SDPA causal prefill of every layer, layers read their own
                         slice
The paper prints no worked numeric example of this path, so beyond those pins the
values are unpinned by the paper itself.
"""
from .plan import build_plan            # noqa: F401
from .rope import rotate                # noqa: F401
from .link import link_kv, link_kv_unshifted, position_fresh, to_slots     # noqa: F401
from .attend import attend, attend_loops, attend_unshifted  # noqa: F401
from .decode import decode_attend       # noqa: F401
from .select import k_distance, top_tokens, top_counts  # noqa: F401
from .store import ChunkStore            # noqa: F401
from .pipeline import plan_with_lookup, prefill_layers  # noqa: F401
