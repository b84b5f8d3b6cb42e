// One kernel table of libenec (see enec_kernels.hpp): all instances of one direction for one
// element format.  ENEC_DT and ENEC_DIR come from the command line.
#include "enec_kernels.hpp"

#if !defined(ENEC_DT) || !defined(ENEC_DIR)
#error "compile with -DENEC_DT=0|1|2 -DENEC_DIR=0|1"
#endif

namespace enec {
namespace {

// every (m, a = n - m) with 1 <= m + a <= NMAX, NMAX = width of the format's exponent field
template <int M, int A, int DT> struct Pick {
    static constexpr int NMAX = (int)exponent_bits(DT);
#if ENEC_DIR == 0
    static CompressFn get(int m, int a)
    {
        if (m == M && a == A) return &compress_kernel<M, A, DT>;
#else
    static DecompressFn get(int m, int a)
    {
        if (m == M && a == A) return &decompress_kernel<M, A, DT>;
#endif
        if constexpr (A < NMAX - M) return Pick<M, A + 1, DT>::get(m, a);
        else if constexpr (M < NMAX) return Pick<M + 1, 0, DT>::get(m, a);
        else return nullptr;
    }
};

}  // namespace

#if ENEC_DIR == 0
#if ENEC_DT == 0
CompressFn pick_compress_bf16(int m, int a) { return Pick<0, 1, DT_BF16>::get(m, a); }
#elif ENEC_DT == 1
CompressFn pick_compress_fp16(int m, int a) { return Pick<0, 1, DT_FP16>::get(m, a); }
#else
CompressFn pick_compress_fp32(int m, int a) { return Pick<0, 1, DT_FP32>::get(m, a); }
#endif
#else
#if ENEC_DT == 0
DecompressFn pick_decompress_bf16(int m, int a) { return Pick<0, 1, DT_BF16>::get(m, a); }
#elif ENEC_DT == 1
DecompressFn pick_decompress_fp16(int m, int a) { return Pick<0, 1, DT_FP16>::get(m, a); }
#else
DecompressFn pick_decompress_fp32(int m, int a) { return Pick<0, 1, DT_FP32>::get(m, a); }
#endif
#endif

}  // namespace enec
