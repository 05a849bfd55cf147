"""Test infrastructure only: the fp64 CPU oracle.  Never imported by the product path."""
