// Epilogue shared by the NT GEMM kernels: what happens to one accumulator element.
#pragma once
#include "slide_internal.h"

namespace sl {

template <typename T, typename RS>
__device__ __forceinline__ void epi_store_mode(int mode, const GemmNT& g, long long m, int n, float acc) {
  switch (mode) {
    case EPI_PLAIN:
      ((T*)g.out)[m * g.ldc + n] = from_f<T>(acc);
      break;
    case EPI_BIAS:
      ((T*)g.out)[m * g.ldc + n] = from_f<T>(acc + g.bias[n]);
      break;
    case EPI_BIAS_RESID:
      ((RS*)g.out)[m * g.ldc + n] = from_f<RS>(acc + g.bias[n] + to_f(((const RS*)g.resid)[m * g.ldr + n]));
      break;
    case EPI_BIAS_GELU: {
      float gl, dg;
      gelu_both(acc + g.bias[n], &gl, &dg);
      ((T*)g.out)[m * g.ldc + n] = from_f<T>(gl);
      ((typename dgelu_store<T>::type*)g.out2)[m * g.ldc2 + n] = dgelu_store<T>::put(dg);
      break;
    }
    case EPI_DGELU:
      ((T*)g.out)[m * g.ldc + n] =
          from_f<T>(acc * dgelu_store<T>::get(((const typename dgelu_store<T>::type*)g.pre)[m * g.ldpre + n]));
      break;
    case EPI_PATCH: {
      long long mm = g.cmap(m);
      int tok = 1 + (int)(m % g.cmap.g2);
      ((RS*)g.out)[mm * g.ldc + n] = from_f<RS>(acc + g.bias[n] + g.pos[(size_t)tok * g.N + n]);
      break;
    }
  }
}

template <typename T, typename RS>
__device__ __forceinline__ void epi_store(const GemmNT& g, long long m, int n, float acc) {
  epi_store_mode<T, RS>(g.epi, g, m, n, acc);
}

}  // namespace sl
