/*
 * pkv_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * Slow, plain CPU reference for the two operations of the library: decode
 * attention over a paged KV pool and the block copy of the preemption swap
 * path.  Everything is computed in fp64 straight from the definition; there is
 * no blocking, no online softmax, no reordering.  It shares no code, header or
 * table with the GPU implementation and takes only host pointers.
 *
 * What is computed and where it comes from (arXiv 2602.07878):
 *  - Sec. 2.2 "KV-Cache": the cache is cut into fixed-size blocks that are
 *    non-contiguous in physical memory -> a per-sequence table of physical
 *    block ids; logical token t lives in table entry t / block_size at slot
 *    t % block_size.
 *  - Sec. 2.1 / Sec. 4.2: each decode step attends from the one new query to
 *    the K/V of all tokens so far (the whole history is streamed every step).
 *    The paper prints no attention formula; the standard scaled dot-product
 *    attention of its reference [attention] is used:
 *        s_t = scale * sum_d q_d K_{t,d},  w = softmax(s),  out = sum_t w_t V_t.
 *  - Sec. 5.1.2 "Swapping": a victim's blocks are copied out of the pool and
 *    later copied back (to other physical blocks) -> a per-(plane, block)
 *    memcpy driven by a list of (source block, destination block) pairs.
 *
 * Pins (tests/test_oracle_pins.py): 1-token context, identical keys, block
 * placement permutation, token-order permutation, weight sum / convex hull,
 * key shift invariance, one-hot limit, GQA = replicated MHA, split-merge
 * algebra, a library attention routine in fp64, exact-rational brute force on
 * tiny inputs, NaN poison outside the defined reads; for the copy: identity,
 * permutation and inverse, round trip, untouched bytes; for the 8-bit pools: all
 * 256 codes against a library conversion and the format's closed forms, the
 * dequantisation factors against the same call on pre-scaled wider pools.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F8E4M3 = 2 };

/* bfloat16 = the upper 16 bits of an IEEE-754 binary32: widening is exact. */
static double bf16_bits_to_double(uint16_t bits) {
  uint32_t w = ((uint32_t)bits) << 16;
  float f;
  memcpy(&f, &w, sizeof f);
  return (double)f;
}

/*
 * 8-bit float E4M3 of the OCP 8-bit floating point specification: 1 sign bit, 4
 * exponent bits (bias 7), 3 mantissa bits; exponent field 0 holds the
 * subnormals m/8 * 2^-6; there are no infinities and the one NaN pattern per
 * sign is S.1111.111, so the largest magnitude is S.1111.110 = 1.75 * 2^8 = 448.
 */
static double f8e4m3_bits_to_double(uint8_t code) {
  const int sign = code >> 7, e = (code >> 3) & 15, m = code & 7;
  if (e == 15 && m == 7) return NAN;
  const double mag = e == 0 ? ldexp((double)m / 8.0, -6) : ldexp(1.0 + (double)m / 8.0, e - 7);
  return sign ? -mag : mag;
}

static double load_elem(const void* base, int64_t index, int dtype) {
  if (dtype == ORC_BF16) return bf16_bits_to_double(((const uint16_t*)base)[index]);
  if (dtype == ORC_F8E4M3) return f8e4m3_bits_to_double(((const uint8_t*)base)[index]);
  return (double)((const float*)base)[index];
}

/*
 * Decode attention, one call = all sequences and query heads.
 *   q            [B][Hq][D]                         (dtype)
 *   k_pool       element (b,g,s,d) at b*ksb + g*ksh + s*kst + d   (dtype)
 *   v_pool       same with vsb, vsh, vst
 *   block_tables [B][max_blocks_per_seq] int32
 *   context_lens [B] int32  (n_i counts every token whose K/V is in the pool)
 *   out          [B][Hq][D] double
 *   weights_out  optional [B][Hq][max_ctx] double: softmax weights (tests)
 * Returns 0, or a negative number for an index that leaves the pool/table.
 */
int orc_paged_decode_attention_kv(
    int B, int Hq, int Hkv, int D, int block_size, int num_pool_blocks,
    int max_blocks_per_seq, int q_dtype, int kv_dtype, float k_scale, float v_scale,
    int64_t ksb, int64_t ksh, int64_t kst,
    int64_t vsb, int64_t vsh, int64_t vst, const void* q, const void* k_pool,
    const void* v_pool, const int32_t* block_tables,
    const int32_t* context_lens, float scale, double* out, double* weights_out,
    int max_ctx);

/* q and the pools in one element type, stored values taken as they are. */
int orc_paged_decode_attention(
    int B, int Hq, int Hkv, int D, int block_size, int num_pool_blocks,
    int max_blocks_per_seq, int dtype, int64_t ksb, int64_t ksh, int64_t kst,
    int64_t vsb, int64_t vsh, int64_t vst, const void* q, const void* k_pool,
    const void* v_pool, const int32_t* block_tables,
    const int32_t* context_lens, float scale, double* out, double* weights_out,
    int max_ctx) {
  return orc_paged_decode_attention_kv(B, Hq, Hkv, D, block_size, num_pool_blocks, max_blocks_per_seq,
                                       dtype, dtype, 1.0f, 1.0f, ksb, ksh, kst, vsb, vsh, vst, q, k_pool,
                                       v_pool, block_tables, context_lens, scale, out, weights_out, max_ctx);
}

/*
 * The same with the pools in their own element type (a quantised KV cache: the
 * time model of Sec. 4.2 charges sizeof(T) bytes per cached element) and a
 * dequantisation factor per pool: K_t[d] = k_scale * stored value, V likewise.
 * Strides count pool elements.
 */
int orc_paged_decode_attention_kv(
    int B, int Hq, int Hkv, int D, int block_size, int num_pool_blocks,
    int max_blocks_per_seq, int q_dtype, int kv_dtype, float k_scale, float v_scale,
    int64_t ksb, int64_t ksh, int64_t kst,
    int64_t vsb, int64_t vsh, int64_t vst, const void* q, const void* k_pool,
    const void* v_pool, const int32_t* block_tables,
    const int32_t* context_lens, float scale, double* out, double* weights_out,
    int max_ctx) {
  if (Hkv <= 0 || Hq % Hkv != 0) return -1;
  const int G = Hq / Hkv;
  int status = 0;

#pragma omp parallel for collapse(2) schedule(dynamic, 1)
  for (int i = 0; i < B; ++i) {
    for (int h = 0; h < Hq; ++h) {
      const int n = context_lens[i];
      double* o = out + ((int64_t)i * Hq + h) * D;
      for (int d = 0; d < D; ++d) o[d] = 0.0;
      if (n <= 0) continue; /* empty context: zero row, nothing is read */
      if ((n + block_size - 1) / block_size > max_blocks_per_seq) {
#pragma omp atomic write
        status = -2;
        continue;
      }
      const int g = h / G; /* contiguous groups of G query heads per KV head */

      /* 1. gather the n rows of K and V contiguously, exactly, as fp64 */
      double* Kc = (double*)malloc(sizeof(double) * (size_t)n * D);
      double* Vc = (double*)malloc(sizeof(double) * (size_t)n * D);
      double* s = (double*)malloc(sizeof(double) * (size_t)n);
      int bad = 0;
      for (int t = 0; t < n; ++t) {
        const int blk = block_tables[(int64_t)i * max_blocks_per_seq + t / block_size];
        const int slot = t % block_size;
        if (blk < 0 || blk >= num_pool_blocks) {
          bad = 1;
          break;
        }
        const int64_t kbase = blk * ksb + g * ksh + slot * kst;
        const int64_t vbase = blk * vsb + g * vsh + slot * vst;
        for (int d = 0; d < D; ++d) {
          Kc[(int64_t)t * D + d] = (double)k_scale * load_elem(k_pool, kbase + d, kv_dtype);
          Vc[(int64_t)t * D + d] = (double)v_scale * load_elem(v_pool, vbase + d, kv_dtype);
        }
      }
      if (bad) {
#pragma omp atomic write
        status = -3;
        free(Kc); free(Vc); free(s);
        continue;
      }

      /* 2. scores: plain left-to-right dot product, then the scale */
      const int64_t qbase = ((int64_t)i * Hq + h) * D;
      for (int t = 0; t < n; ++t) {
        double acc = 0.0;
        for (int d = 0; d < D; ++d)
          acc += load_elem(q, qbase + d, q_dtype) * Kc[(int64_t)t * D + d];
        s[t] = (double)scale * acc;
      }

      /* 3. softmax with the maximum subtracted */
      double m = s[0];
      for (int t = 1; t < n; ++t) if (s[t] > m) m = s[t];
      double Z = 0.0;
      for (int t = 0; t < n; ++t) { s[t] = exp(s[t] - m); Z += s[t]; }
      for (int t = 0; t < n; ++t) s[t] /= Z;
      if (weights_out) {
        double* w = weights_out + ((int64_t)i * Hq + h) * max_ctx;
        for (int t = 0; t < n && t < max_ctx; ++t) w[t] = s[t];
      }

      /* 4. weighted sum of the value rows */
      for (int t = 0; t < n; ++t)
        for (int d = 0; d < D; ++d) o[d] += s[t] * Vc[(int64_t)t * D + d];

      free(Kc); free(Vc); free(s);
    }
  }
  return status;
}

/*
 * Block copy of the swap path: for every plane p and pair j,
 *   dst[p*dst_plane_stride + d_j*block_bytes .. +block_bytes) =
 *   src[p*src_plane_stride + s_j*block_bytes .. +block_bytes).
 * mapping is [n_pairs][2] = (s_j, d_j).  Returns 0, or negative when a pair
 * leaves its plane.
 */
int orc_kv_block_swap(int num_planes, int64_t block_bytes,
                      int64_t src_plane_stride, int64_t dst_plane_stride,
                      int src_num_blocks, int dst_num_blocks,
                      const uint8_t* src, uint8_t* dst, const int32_t* mapping,
                      int n_pairs) {
  for (int j = 0; j < n_pairs; ++j) {
    const int s = mapping[2 * j], d = mapping[2 * j + 1];
    if (s < 0 || s >= src_num_blocks || d < 0 || d >= dst_num_blocks) return -1;
  }
#pragma omp parallel for schedule(static)
  for (int64_t pj = 0; pj < (int64_t)num_planes * n_pairs; ++pj) {
    const int p = (int)(pj / n_pairs), j = (int)(pj % n_pairs);
    const int64_t s = mapping[2 * j], d = mapping[2 * j + 1];
    memcpy(dst + p * dst_plane_stride + d * block_bytes,
           src + p * src_plane_stride + s * block_bytes, (size_t)block_bytes);
  }
  return 0;
}

/*
 * KV append (arXiv 2602.07878, Sec. 2.2 "KV-Cache": the K and V vectors of the
 * token generated in a step are added to the request's cache).  context_lens
 * already counts the new token, so for every sequence i with n_i >= 1 the rows
 * k_new[i][g][:] and v_new[i][g][:] go to token position n_i - 1:
 * block block_tables[i][(n_i-1)/bs], slot (n_i-1)%bs, every KV head g.
 * Sequences with n_i == 0 are skipped.  Strides are in elements, eb = bytes
 * per element.  Returns 0, or negative for an index outside table or pool.
 */
int orc_kv_append(int B, int Hkv, int D, int bs, int nblk, int maxb, int eb,
                  int64_t ksb, int64_t ksh, int64_t kst,
                  int64_t vsb, int64_t vsh, int64_t vst,
                  const uint8_t* k_new, const uint8_t* v_new,
                  uint8_t* k_pool, uint8_t* v_pool,
                  const int32_t* bt, const int32_t* cl) {
  for (int i = 0; i < B; ++i) {
    const int n = cl[i];
    if (n < 0) return -1;
    if (n == 0) continue;
    const int pos = n - 1;
    if (pos / bs >= maxb) return -2;
    const int64_t blk = bt[(int64_t)i * maxb + pos / bs];
    if (blk < 0 || blk >= nblk) return -3;
    const int slot = pos % bs;
    for (int g = 0; g < Hkv; ++g) {
      const size_t row = (size_t)D * eb;
      memcpy(k_pool + (blk * ksb + g * ksh + slot * kst) * eb,
             k_new + ((int64_t)i * Hkv + g) * row, row);
      memcpy(v_pool + (blk * vsb + g * vsh + slot * vst) * eb,
             v_new + ((int64_t)i * Hkv + g) * row, row);
    }
  }
  return 0;
}

int orc_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
  extern int omp_get_max_threads(void);
  n = omp_get_max_threads();
#endif
  return n;
}
