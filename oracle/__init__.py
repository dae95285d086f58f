"""TEST INFRASTRUCTURE: the CPU oracle.  Never imported by the product package."""
