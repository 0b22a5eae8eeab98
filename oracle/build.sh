#!/bin/sh
# Builds the CPU oracle (test infrastructure) into oracle/libziplm_oracle.so.
set -e
cd "$(dirname "$0")"
gcc -O3 -march=x86-64-v3 -fopenmp -fPIC -shared -std=c99 -Wall -Wextra \
    -o libziplm_oracle.so ziplm_oracle.c -lm
