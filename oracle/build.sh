#!/bin/sh
# Builds the CPU oracle (test infrastructure) as a shared library.
set -e
cd "$(dirname "$0")"
gcc -O2 -std=c99 -Wall -Wextra -ffp-contract=off -fPIC -shared \
    -o libqsgd_oracle.so qsgd_oracle.c -lm
