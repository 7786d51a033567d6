#!/bin/bash
# usage: build.sh <source dir with the .hip/.cpp files> <output dir> [extra compiler flags]
# Translates the HIP sources, compiles them with the driver for the host under ASan + UBSan.
set -e
here=$(cd "$(dirname "$0")" && pwd)
src=$1; out=$2; shift 2
mkdir -p "$out"
for f in ccdc.hip pipeline.hip node.hip noalloc.hip map.hip; do
  python3 "$here/translate.py" "$src/$f" "$out/${f%.hip}.cpp"
done
python3 "$here/translate.py" "$src/common.hpp" "$out/common.hpp"     # found first by the translated sources
CXX=${SHIM_CXX:-/opt/rocm/lib/llvm/bin/clang++}
FLAGS="-std=c++20 -O0 -gline-tables-only -fno-omit-frame-pointer -fsanitize=address,undefined -fno-sanitize-recover=undefined -pthread -I $here -I $here/../../include -I $src -Wno-unknown-attributes"
pids=""
for f in "$out/ccdc.cpp" "$out/pipeline.cpp" "$out/node.cpp" "$out/noalloc.cpp" "$out/map.cpp" "$src/plan.cpp" "$here/shim.cpp" "$here/driver.cpp"; do
  $CXX $FLAGS "$@" -c "$f" -o "$out/$(basename "$f").o" &
  pids="$pids $!"
done
for p in $pids; do wait $p; done
$CXX $FLAGS "$out"/*.o -o "$out/driver"
echo "$out/driver"
