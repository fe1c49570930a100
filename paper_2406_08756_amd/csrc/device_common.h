// Device-side helpers shared by the HIP kernels: storage-type loads/stores in
// 16-byte vectors, wavefront reductions, and the Philox dropout generator.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lynx {

typedef __bf16 bf16_t;
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Two floats -> packed bf16 pair, round to nearest even (v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  floatx2_t f = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
}

__device__ __forceinline__ float round_to_storage(float v, const float*) { return v; }
__device__ __forceinline__ float round_to_storage(float v, const bf16_t*) {
  return bf16_lo(pack_bf16(v, 0.f));
}

// 8 consecutive elements <-> 8 floats.
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w;
  v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float (&v)[8]) {
  const uint4 r = *reinterpret_cast<const uint4*>(p);
  v[0] = bf16_lo(r.x); v[1] = bf16_hi(r.x); v[2] = bf16_lo(r.y); v[3] = bf16_hi(r.y);
  v[4] = bf16_lo(r.z); v[5] = bf16_hi(r.z); v[6] = bf16_lo(r.w); v[7] = bf16_hi(r.w);
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t* p, const float (&v)[8]) {
  uint4 r;
  r.x = pack_bf16(v[0], v[1]); r.y = pack_bf16(v[2], v[3]);
  r.z = pack_bf16(v[4], v[5]); r.w = pack_bf16(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = r;
}

// The same stores with the streaming hint: for a tensor nothing reads again soon, so that it
// does not push a tensor the next kernel reads out of the caches.
typedef unsigned int uint32x4_t __attribute__((ext_vector_type(4)));
typedef float float32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store8_streaming(float* p, const float (&v)[8]) {
  __builtin_nontemporal_store(float32x4_t{v[0], v[1], v[2], v[3]}, reinterpret_cast<float32x4_t*>(p));
  __builtin_nontemporal_store(float32x4_t{v[4], v[5], v[6], v[7]}, reinterpret_cast<float32x4_t*>(p + 4));
}
__device__ __forceinline__ void store8_streaming(bf16_t* p, const float (&v)[8]) {
  const uint32x4_t r = {pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7])};
  __builtin_nontemporal_store(r, reinterpret_cast<uint32x4_t*>(p));
}

// 8 storage elements as loaded, before conversion (keeps loads cheap to batch).
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> { uint4 v; };
template <> struct Raw8<float> { float4 lo, hi; };
__device__ __forceinline__ void load_raw(const bf16_t* p, Raw8<bf16_t>& r) {
  r.v = *reinterpret_cast<const uint4*>(p);
}
__device__ __forceinline__ void load_raw(const float* p, Raw8<float>& r) {
  r.lo = *reinterpret_cast<const float4*>(p);
  r.hi = *reinterpret_cast<const float4*>(p + 4);
}
__device__ __forceinline__ void unpack(const Raw8<bf16_t>& r, float (&v)[8]) {
  v[0] = bf16_lo(r.v.x); v[1] = bf16_hi(r.v.x); v[2] = bf16_lo(r.v.y); v[3] = bf16_hi(r.v.y);
  v[4] = bf16_lo(r.v.z); v[5] = bf16_hi(r.v.z); v[6] = bf16_lo(r.v.w); v[7] = bf16_hi(r.v.w);
}
__device__ __forceinline__ void unpack(const Raw8<float>& r, float (&v)[8]) {
  v[0] = r.lo.x; v[1] = r.lo.y; v[2] = r.lo.z; v[3] = r.lo.w;
  v[4] = r.hi.x; v[5] = r.hi.y; v[6] = r.hi.z; v[7] = r.hi.w;
}

// Loads with the non-temporal hint, for a tensor the kernel reads once and nothing reads again
// soon: the lines do not displace what the next kernel will want from the caches.
__device__ __forceinline__ void load_raw_streaming(const bf16_t* p, Raw8<bf16_t>& r) {
  const uint32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const uint32x4_t*>(p));
  r.v = make_uint4(v[0], v[1], v[2], v[3]);
}
__device__ __forceinline__ void load_raw_streaming(const float* p, Raw8<float>& r) {
  const float32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const float32x4_t*>(p));
  const float32x4_t b = __builtin_nontemporal_load(reinterpret_cast<const float32x4_t*>(p + 4));
  r.lo = make_float4(a[0], a[1], a[2], a[3]);
  r.hi = make_float4(b[0], b[1], b[2], b[3]);
}
template <typename T>
__device__ __forceinline__ void load8_streaming(const T* p, float (&v)[8]) {
  Raw8<T> r;
  load_raw_streaming(p, r);
  unpack(r, v);
}

// Makes the compiler forget what it derived from r, so values unpacked from it earlier are
// recomputed from the (smaller) storage form instead of being kept in registers.
__device__ __forceinline__ void forget(Raw8<bf16_t>& r) {
  asm volatile("" : "+v"(r.v.x), "+v"(r.v.y), "+v"(r.v.z), "+v"(r.v.w));
}
__device__ __forceinline__ void forget(Raw8<float>&) {}

__device__ __forceinline__ float load1(const float* p) { return *p; }
__device__ __forceinline__ float load1(const bf16_t* p) {
  return __uint_as_float(static_cast<uint32_t>(*reinterpret_cast<const uint16_t*>(p)) << 16);
}
__device__ __forceinline__ void store1(float* p, float v) { *p = v; }
__device__ __forceinline__ void store1(bf16_t* p, float v) {
  *reinterpret_cast<uint16_t*>(p) = static_cast<uint16_t>(pack_bf16(v, 0.f) & 0xFFFFu);
}

// Butterfly reductions over the 64 lanes of a wavefront: every lane ends with
// the result, and the combination order is fixed (deterministic).
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}
// Sum over each aligned group of 8 lanes in the tree order ((v0 + v1) + (v2 + v3)) + ((v4 + v5)
// + (v6 + v7)); every lane of the group gets the same bits (addition commutes).  Data-parallel
// lane permutes inside the vector ALU: no trip through the LDS crossbar.
template <int CTRL>
__device__ __forceinline__ float lane_permute(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xF, 0xF, true));
}
__device__ __forceinline__ float group8_sum(float v) {
  v += lane_permute<0xB1>(v);   // quad_perm [1, 0, 3, 2]: lane ^ 1
  v += lane_permute<0x4E>(v);   // quad_perm [2, 3, 0, 1]: lane ^ 2
  v += lane_permute<0x141>(v);  // row_half_mirror: lane 7 - i, a lane of the other quad (all four hold its sum)
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

// ---------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  One call yields four 32-bit words =
// eight 16-bit fields = the dropout decisions of eight consecutive elements.
// ---------------------------------------------------------------------------
struct DropoutKey {
  uint32_t key0, key1;        // seed lo, hi
  uint32_t stream0, stream1;  // (layer_id << 2 | site), step
  uint32_t threshold;         // keep iff field >= threshold (floor(p * 65536))
  float scale;                // 1 / (1 - p)
};

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = static_cast<uint64_t>(0xD2511F53u) * c0;
    const uint64_t p1 = static_cast<uint64_t>(0xCD9E8D57u) * c2;
    const uint32_t n0 = static_cast<uint32_t>(p1 >> 32) ^ c1 ^ k0;
    const uint32_t n2 = static_cast<uint32_t>(p0 >> 32) ^ c3 ^ k1;
    c1 = static_cast<uint32_t>(p1);
    c3 = static_cast<uint32_t>(p0);
    c0 = n0;
    c2 = n2;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return make_uint4(c0, c1, c2, c3);
}

// Keep-bits (bit l = element 8*group + l is kept) of one group of 8 elements.
__device__ __forceinline__ uint32_t dropout_keep8(const DropoutKey& k, uint64_t group) {
  const uint4 w = philox4x32_10(static_cast<uint32_t>(group), static_cast<uint32_t>(group >> 32),
                                k.stream0, k.stream1, k.key0, k.key1);
  const uint32_t t = k.threshold;
  uint32_t m = 0;
  m |= ((w.x & 0xFFFFu) >= t) ? 1u : 0u;
  m |= ((w.x >> 16) >= t) ? 2u : 0u;
  m |= ((w.y & 0xFFFFu) >= t) ? 4u : 0u;
  m |= ((w.y >> 16) >= t) ? 8u : 0u;
  m |= ((w.z & 0xFFFFu) >= t) ? 16u : 0u;
  m |= ((w.z >> 16) >= t) ? 32u : 0u;
  m |= ((w.w & 0xFFFFu) >= t) ? 64u : 0u;
  m |= ((w.w >> 16) >= t) ? 128u : 0u;
  return m;
}

// v[l] = keep(l) ? v[l] * scale : 0 for the 8 elements of one group, straight from
// the 16-bit fields (no intermediate bit mask).
__device__ __forceinline__ void dropout_apply8(const DropoutKey& k, uint64_t group, float (&v)[8]) {
  const uint4 w = philox4x32_10(static_cast<uint32_t>(group), static_cast<uint32_t>(group >> 32),
                                k.stream0, k.stream1, k.key0, k.key1);
  const uint32_t t = k.threshold;
  const float s = k.scale;
  v[0] = ((w.x & 0xFFFFu) >= t) ? v[0] * s : 0.0f;
  v[1] = ((w.x >> 16) >= t) ? v[1] * s : 0.0f;
  v[2] = ((w.y & 0xFFFFu) >= t) ? v[2] * s : 0.0f;
  v[3] = ((w.y >> 16) >= t) ? v[3] * s : 0.0f;
  v[4] = ((w.z & 0xFFFFu) >= t) ? v[4] * s : 0.0f;
  v[5] = ((w.z >> 16) >= t) ? v[5] * s : 0.0f;
  v[6] = ((w.w & 0xFFFFu) >= t) ? v[6] * s : 0.0f;
  v[7] = ((w.w >> 16) >= t) ? v[7] * s : 0.0f;
}

}  // namespace lynx
