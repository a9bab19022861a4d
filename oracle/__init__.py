"""CPU fp64 oracle for hierarchical document attention.  Test infrastructure only: nothing in
the product path may import this package."""
