"""CPU oracle of the FF-INT8 layer-local train step.  Test infrastructure only:
imported by tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg."""
