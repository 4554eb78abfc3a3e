"""fp64 CPU oracle for the PBS-Attn prefill path.  Test infrastructure only: see pbs_oracle.c."""
