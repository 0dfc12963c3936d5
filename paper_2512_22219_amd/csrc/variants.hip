// Instantiates the kernels.  Built once per specialised set with -DMPK_VARIANT_INDEX=i (the sets
// compile in parallel, each in a translation unit of its own); without the definition every set is
// instantiated here.
#include "kernels.h"

namespace mpk {

template <int I> struct VariantParams;
#define MPK_PARAMS(I, D, G, N, M)                    \
  template <> struct VariantParams<I> {              \
    static constexpr int d = D, grp = G, nb = N;     \
    static constexpr bool moe = M;                   \
  };
MPK_VARIANT_LIST(MPK_PARAMS)
#undef MPK_PARAMS

template <int I>
static const KernelVariant* make_variant() {
  using P = VariantParams<I>;
  constexpr bool split = P::nb == 8;   // matrix-core bodies: one kernel per launch path
  // kernel sets compiled for a model shape: several steps are issued as a launch per step
  void (*run_step)(StepArgs) = nullptr;
  if constexpr (P::nb == 1 || P::nb == 9) run_step = mpk_mega_kernel<P::d, P::grp, P::nb, P::moe, 0, true>;
  if constexpr (P::nb == 8) run_step = mpk_mega_kernel<P::d, P::grp, P::nb, P::moe, 1, true>;
  static const KernelVariant v = {P::d, P::grp, P::nb, P::moe, mpk_mega_kernel<P::d, P::grp, P::nb, P::moe, split ? 1 : 0>,
                                  mpk_op_kernel<P::d, P::grp, P::nb, P::moe>, mpk_loop_kernel<P::d, P::grp, P::nb, P::moe>,
                                  mpk_mega_kernel<P::d, P::grp, P::nb, P::moe, split ? 2 : 0>, run_step};
  return &v;
}

#define MPK_DEFINE_VARIANT(I) \
  const KernelVariant* kernel_variant_##I() { return make_variant<I>(); }

#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 0
MPK_DEFINE_VARIANT(0)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 1
MPK_DEFINE_VARIANT(1)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 2
MPK_DEFINE_VARIANT(2)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 3
MPK_DEFINE_VARIANT(3)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 4
MPK_DEFINE_VARIANT(4)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 5
MPK_DEFINE_VARIANT(5)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 6
MPK_DEFINE_VARIANT(6)
#endif
#if !defined(MPK_VARIANT_INDEX) || MPK_VARIANT_INDEX == 7
MPK_DEFINE_VARIANT(7)
#endif

}  // namespace mpk
