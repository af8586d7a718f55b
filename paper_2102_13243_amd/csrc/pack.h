// Small fixed-width channel vectors: V adjacent channels of storage type T moved with one
// memory instruction (16 bytes for float x4 and bf16 x8) and read/written as fp32.
#pragma once
#include "s4tf_internal.h"

namespace s4tf {

template <typename T, int V> struct Pack;  // V channels of type T
template <> struct Pack<float, 4> {
  float4 d;
  __device__ float get(int i) const { return i == 0 ? d.x : i == 1 ? d.y : i == 2 ? d.z : d.w; }
  __device__ void set(int i, float v) { if (i == 0) d.x = v; else if (i == 1) d.y = v; else if (i == 2) d.z = v; else d.w = v; }
};
template <> struct Pack<float, 1> {
  float d;
  __device__ float get(int) const { return d; }
  __device__ void set(int, float v) { d = v; }
};
template <> struct Pack<bf16_t, 8> {
  uint4 d;
  __device__ float get(int i) const {
    uint32_t w = i < 2 ? d.x : i < 4 ? d.y : i < 6 ? d.z : d.w;
    return bf16_to_f32((bf16_t)((i & 1) ? (w >> 16) : (w & 0xffffu)));
  }
  __device__ void set(int i, float v) {
    uint32_t b = f32_to_bf16(v);
    uint32_t& w = i < 2 ? d.x : i < 4 ? d.y : i < 6 ? d.z : d.w;
    w = (i & 1) ? ((w & 0xffffu) | (b << 16)) : ((w & 0xffff0000u) | b);
  }
};
template <> struct Pack<bf16_t, 1> {
  bf16_t d;
  __device__ float get(int) const { return bf16_to_f32(d); }
  __device__ void set(int, float v) { d = f32_to_bf16(v); }
};

// A whole vector from V fp32 values: the bf16 x8 case converts pairs with one instruction each
// (v_cvt_pk_bf16_f32) instead of inserting eight separately converted halves.
template <typename T, int V> __device__ inline Pack<T, V> pack_of(const float (&v)[V]) {
  Pack<T, V> o;
#pragma unroll
  for (int e = 0; e < V; ++e) o.set(e, v[e]);
  return o;
}
template <> __device__ inline Pack<bf16_t, 8> pack_of<bf16_t, 8>(const float (&v)[8]) {
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  Pack<bf16_t, 8> o;
  uint32_t w[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f32x2_t f = {v[2 * i], v[2 * i + 1]};
    w[i] = __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
  }
  o.d = make_uint4(w[0], w[1], w[2], w[3]);
  return o;
}

template <typename T, int V> __device__ inline Pack<T, V> ldp(const T* p) {
  return *reinterpret_cast<const Pack<T, V>*>(p);
}
template <typename T, int V> __device__ inline void stp(T* p, const Pack<T, V>& v) {
  *reinterpret_cast<Pack<T, V>*>(p) = v;
}


template <typename T> struct VecOf;
template <> struct VecOf<float> { static constexpr int V = 4; };
template <> struct VecOf<bf16_t> { static constexpr int V = 8; };

}  // namespace s4tf
