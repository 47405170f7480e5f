// Prints Philox4x32-10 blocks computed by the counter-based engine that ships in PyTorch's ATen
// headers (a library routine, independent of this repository), for the oracle's pin test.
// usage: prog seed subsequence offset [seed subsequence offset ...]
// ATen's engine: key = (seed lo, seed hi), counter = (offset lo, offset hi, subsequence lo, subsequence hi).
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  for (int i = 1; i + 2 < argc; i += 3) {
    unsigned long long seed = strtoull(argv[i], 0, 0), subseq = strtoull(argv[i+1], 0, 0), off = strtoull(argv[i+2], 0, 0);
    at::philox_engine e(seed, subseq, off);
    unsigned a = e(), b = e(), c = e(), d = e();
    printf("%08x %08x %08x %08x\n", a, b, c, d);
  }
  return 0;
}
