"""CPU oracle for the backup-worker Sync-SGD step.  Test infrastructure only:
only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may use it."""
