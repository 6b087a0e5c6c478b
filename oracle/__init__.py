"""CPU oracle for SpecASR tree verification -- TEST INFRASTRUCTURE, not the product.

Two independent forms:

* ``tree``   : ctypes wrapper around ``specasr_oracle.c`` (the tree algorithm in
               fp64, step by step: ancestor mask, depth-keyed positions, greedy
               acceptance; paper Sec. II-B and Sec. IV-C).
* ``sparse_tree`` : the draft-side control of a round (adaptive truncation, recycling merge,
               two-pass sparse tree; paper Sec. IV-A/B/C) as plain Python over a recorded draft
               read-out.
* ``form_s`` : a numpy fp64 causal decoder with no KV cache and no mask beyond
               the causal one -- the brute-force definition every tree node's
               logits must equal (speculative decoding is lossless, Sec. II-B).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this
package.  It shares no code with the HIP library.
"""
from .tree import (OracleModel, build_oracle, tree_meta, accept, top2, rmsnorm, rope, softmax,
                   silu, num_threads)
from . import form_s, sparse_tree

__all__ = ["OracleModel", "build_oracle", "tree_meta", "accept", "top2", "rmsnorm", "rope",
           "softmax", "silu", "num_threads", "form_s", "sparse_tree"]
