"""CPU oracle of the W4A16 / bf16 linear path.  Test infrastructure only: see dmr_oracle.c."""
