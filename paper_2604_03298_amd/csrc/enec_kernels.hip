// One kernel table of libenec (see enec_kernels.hpp): all instances of one direction for one
// element format and one group length.  ENEC_DT, ENEC_LPG and ENEC_DIR come from the command line.
#include "enec_kernels.hpp"

#if !defined(ENEC_DT) || !defined(ENEC_DIR) || !defined(ENEC_LPG)
#error "compile with -DENEC_DT=0|1|2 -DENEC_LPG=1|2|4 -DENEC_DIR=0|1"
#endif

namespace enec {
namespace {

// every (m, a = n - m) with 1 <= m + a <= NMAX, NMAX = width of the format's exponent field
template <int M, int A> struct Pick {
    static constexpr int NMAX = (int)exponent_bits(ENEC_DT);
#if ENEC_DIR == 0
    static CompressFn get(int m, int a)
    {
        if (m == M && a == A) return &compress_kernel<M, A, ENEC_DT, ENEC_LPG>;
#else
    static DecompressFn get(int m, int a)
    {
        if (m == M && a == A) return &decompress_kernel<M, A, ENEC_DT, ENEC_LPG>;
#endif
        if constexpr (A < NMAX - M) return Pick<M, A + 1>::get(m, a);
        else if constexpr (M < NMAX) return Pick<M + 1, 0>::get(m, a);
        else return nullptr;
    }
};

}  // namespace

#define ENEC_CAT2(a, b, c, d) a##b##c##d
#define ENEC_CAT(a, b, c, d) ENEC_CAT2(a, b, c, d)
#if ENEC_DIR == 0
CompressFn ENEC_CAT(pick_compress_dt, ENEC_DT, _lpg, ENEC_LPG)(int m, int a) { return Pick<0, 1>::get(m, a); }
#else
DecompressFn ENEC_CAT(pick_decompress_dt, ENEC_DT, _lpg, ENEC_LPG)(int m, int a) { return Pick<0, 1>::get(m, a); }
#endif

}  // namespace enec
