#!/bin/bash
# Builds libkdloss.so for gfx950 next to the sources.
set -e
cd "$(dirname "$0")"
hipcc --offload-arch=gfx950 -O3 -std=c++17 -fPIC -shared \
  -Xclang -target-feature -Xclang -packed-fp32-ops \
  kd_kernels.hip kd_api.hip -o libkdloss.so "$@"
