// Prints 32-bit outputs of rocRAND's Philox4x32-10 engine, run on the host (the engine's
// methods are __host__ __device__).  Used by tests/test_oracle_philox.py as an independent
// implementation of the generator: arguments are seed, subsequence, offset, count; the engine
// takes the seed as key, the subsequence as the upper two counter words and offset / 4 as the
// lower two, and returns the four words of a block in order.
#include <hip/hip_runtime.h>
#include <rocrand/rocrand_philox4x32_10.h>

#include <cstdio>
#include <cstdlib>

int main(int argc, char** argv) {
  if (argc != 5) {
    std::fprintf(stderr, "usage: %s seed subsequence offset count\n", argv[0]);
    return 2;
  }
  const unsigned long long seed = std::strtoull(argv[1], nullptr, 0);
  const unsigned long long subsequence = std::strtoull(argv[2], nullptr, 0);
  const unsigned long long offset = std::strtoull(argv[3], nullptr, 0);
  const long count = std::atol(argv[4]);
  rocrand_device::philox4x32_10_engine engine(seed, subsequence, offset);
  for (long i = 0; i < count; ++i) std::printf("%u\n", engine());
  return 0;
}
