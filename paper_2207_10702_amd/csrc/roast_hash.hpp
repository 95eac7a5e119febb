// Integer side of ROAST: block key -> (offset in M, sign).  Host and device share this one
// implementation inside the library (the CPU oracle has its own, in plain C with % operators).
//
// The map is the Carter-Wegman family stated in roast.h (hash h1 / h2 and sign g of Section 3.1 of
// arXiv 2207.10702).  Every `mod` is a Barrett reduction with a reciprocal prepared once on the
// host, so the device never runs a 64-bit divide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "roast.h"

namespace roast {

// x mod d for any 64-bit x, using mu = floor(2^64 / d) (all-ones when d == 1).
// floor(x*mu / 2^64) is the true quotient or one less, so one conditional subtract finishes it.
struct Barrett {
  uint64_t d;
  uint64_t mu;
};

inline Barrett make_barrett(uint64_t d) {
  Barrett b;
  b.d = d;
  b.mu = (d <= 1) ? ~0ull : (uint64_t)((((unsigned __int128)1) << 64) / d);
  return b;
}

__host__ __device__ inline uint64_t mulhi64(uint64_t a, uint64_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umul64hi(a, b);
#else
  return (uint64_t)(((unsigned __int128)a * b) >> 64);
#endif
}

__host__ __device__ inline uint64_t bmod(uint64_t x, const Barrett& b) {
  uint64_t q = mulhi64(x, b.mu);
  uint64_t r = x - q * b.d;
  return r >= b.d ? r - b.d : r;
}

// Everything a kernel needs to place a block; passed by value as a kernel argument.
struct HashDev {
  Barrett P;      // prime modulus
  Barrett slots;  // number of legal offsets / align
  uint64_t a0, a1, a2, a3;
  uint64_t s0, s1, s2, s3;
  uint32_t align;
  uint32_t use_sign;
};

// block = scalars per block (Z1*Z2 or Z).  Caller has validated m_size >= block, align >= 1.
inline HashDev make_hash_dev(const roast_hash& h, int64_t m_size, int64_t block) {
  HashDev d;
  d.P = make_barrett(h.P);
  d.slots = make_barrett((uint64_t)(m_size - block) / h.align + 1);
  d.a0 = h.a0; d.a1 = h.a1; d.a2 = h.a2; d.a3 = h.a3;
  d.s0 = h.s0; d.s1 = h.s1; d.s2 = h.s2; d.s3 = h.s3;
  d.align = h.align;
  d.use_sign = h.use_sign;
  return d;
}

// (c0*k0 + c1*k1 + c2*k2 + c3) mod P with keys and products reduced first (no 64-bit overflow
// for any P < 2^32).
__host__ __device__ inline uint64_t cw(const Barrett& P, uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3,
                                       uint64_t k0, uint64_t k1, uint64_t k2) {
  uint64_t t0 = bmod(c0 * bmod(k0, P), P);
  uint64_t t1 = bmod(c1 * bmod(k1, P), P);
  uint64_t t2 = bmod(c2 * bmod(k2, P), P);
  return bmod(t0 + t1 + t2 + c3, P);
}

__host__ __device__ inline int64_t block_offset(const HashDev& h, uint64_t k0, uint64_t k1, uint64_t k2) {
  uint64_t u = cw(h.P, h.a0, h.a1, h.a2, h.a3, k0, k1, k2);
  return (int64_t)((uint64_t)h.align * bmod(u, h.slots));
}

// +1 or -1
__host__ __device__ inline int block_sign(const HashDev& h, uint64_t k0, uint64_t k1, uint64_t k2) {
  if (!h.use_sign) return 1;
  uint64_t v = cw(h.P, h.s0, h.s1, h.s2, h.s3, k0, k1, k2);
  return 1 - 2 * (int)(v & 1ull);
}

}  // namespace roast
