// Host-side checker: prints Philox4x32-10 outputs computed by AMD's rocRAND
// engine (an implementation independent of both the oracle's and the HIP
// library's) for counters/keys read from stdin.  Used by the CPU tests only.
// Input lines:  k0 k1 c0 c1 c2 c3   (hex).  Output: four hex words per line.
#include <rocrand/rocrand_philox4x32_10.h>
#include <cstdio>

struct Exposed : public rocrand_device::philox4x32_10_engine {
    __host__ uint4 block(uint4 c, uint2 k) { return this->ten_rounds(c, k); }
};

int main() {
    unsigned k0, k1, c0, c1, c2, c3;
    Exposed e;
    while (scanf("%x %x %x %x %x %x", &k0, &k1, &c0, &c1, &c2, &c3) == 6) {
        uint4 c; c.x = c0; c.y = c1; c.z = c2; c.w = c3;
        uint2 k; k.x = k0; k.y = k1;
        uint4 r = e.block(c, k);
        printf("%08x %08x %08x %08x\n", r.x, r.y, r.z, r.w);
    }
    return 0;
}
