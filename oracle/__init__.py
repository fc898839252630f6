"""CPU oracles for top-k attention decode.  TEST INFRASTRUCTURE ONLY.

`topk_attention_ref` is the NumPy float64 definition; `c_oracle` wraps the plain
C version (same definition, fast enough for million-token caches).  Nothing
under the product package imports this directory.
"""
