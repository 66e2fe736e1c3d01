#!/bin/sh
# Builds the CPU oracle (test infrastructure) into oracle/libsparseloco_oracle.so.
# -ffp-contract=off: the only fused operation is the explicit fmaf.
set -e
cd "$(dirname "$0")"
gcc -O2 -std=c11 -ffp-contract=off -fopenmp -fPIC -shared -Wall -Wextra \
    -o libsparseloco_oracle.so sparseloco_oracle.c -lm
