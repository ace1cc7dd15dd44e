#!/bin/sh
# Builds the CPU oracle (plain g++, no GPU toolchain involved).
set -e
here="$(cd "$(dirname "$0")" && pwd)"
g++ -O2 -std=c++17 -fPIC -shared -frounding-math -fno-fast-math \
    -o "$here/libkvbfp_oracle.so" "$here/kvbfp_oracle.cpp"
