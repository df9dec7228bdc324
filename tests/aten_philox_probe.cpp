// Prints words of PyTorch's own Philox4_32 engine (ATen/core/PhiloxRNGEngine.h),
// an implementation independent of the oracle's, for the cross-check in
// test_oracle_philox.py.  usage: probe seed subsequence offset n_calls
#include <ATen/core/PhiloxRNGEngine.h>
#include <cstdio>
#include <cstdlib>
int main(int argc, char** argv) {
  if (argc != 5) return 2;
  uint64_t seed = strtoull(argv[1], nullptr, 0);
  uint64_t subseq = strtoull(argv[2], nullptr, 0);
  uint64_t offset = strtoull(argv[3], nullptr, 0);
  long n = atol(argv[4]);
  at::Philox4_32 eng(seed, subseq, offset);
  for (long i = 0; i < n; ++i) printf("%u\n", eng());
  return 0;
}
