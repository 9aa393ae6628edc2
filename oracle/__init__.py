"""CPU oracle (fp64 numpy).  Test infrastructure: never imported by the product package."""
