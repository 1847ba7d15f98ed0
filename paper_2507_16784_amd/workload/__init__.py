"""Seeded synthetic inputs shared by the tests, the benchmark and the oracle's
timing leg: reasoning-tree traces with structural marks, initial paging state,
and random Q/K/V tensors.  Holds none of the method's arithmetic."""
