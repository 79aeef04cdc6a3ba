"""CPU oracle of the early-exit decode path.  Test infrastructure only: nothing in the
product package may import this."""
