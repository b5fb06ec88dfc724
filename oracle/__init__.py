"""fp64 CPU oracle of the SWA decode path.  Test infrastructure only."""
