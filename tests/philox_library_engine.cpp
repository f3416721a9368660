// Prints raw outputs of the Philox4x32-10 engine that ships in the installed
// PyTorch headers (a third-party implementation of the published generator),
// for cross-checking the oracle's own implementation.  Host-only; no GPU.
//
// usage: philox_library_engine seed subsequence offset n_blocks
// prints n_blocks lines of four hex words.
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>

int main(int argc, char** argv) {
  if (argc != 5) return 2;
  unsigned long long seed = strtoull(argv[1], nullptr, 0);
  unsigned long long subseq = strtoull(argv[2], nullptr, 0);
  unsigned long long offset = strtoull(argv[3], nullptr, 0);
  unsigned long long n = strtoull(argv[4], nullptr, 0);
  at::philox_engine eng(seed, subseq, offset);
  for (unsigned long long b = 0; b < n; ++b) {
    unsigned x0 = eng(), x1 = eng(), x2 = eng(), x3 = eng();
    printf("%08x %08x %08x %08x\n", x0, x1, x2, x3);
  }
  return 0;
}
