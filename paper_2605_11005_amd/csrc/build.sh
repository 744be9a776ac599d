#!/bin/bash
# Builds libmoe_mi355x.so for gfx950 (run from anywhere; output lands next to the package).
# -Wno-inline-asm: the LDS-DMA loads name M0 in their clobber list on purpose (they set it).
set -e
cd "$(dirname "$0")"
exec hipcc --offload-arch=gfx950 -O3 -std=c++17 -fPIC -shared \
  -Xclang -target-feature -Xclang -packed-fp32-ops -Wno-inline-asm "$@" \
  api.hip route.hip plan.hip rowmove.hip expert_f32.hip expert_bf16.hip router.hip probes.hip alloc.hip -o ../libmoe_mi355x.so
