/* Host-sanitizer leg of the oracle: reads one case from a binary file into heap buffers of
 * exactly the stated sizes (so that AddressSanitizer sees any access outside them), runs one of
 * the oracle's routines and writes the result.  Built by tests/test_sanitizers.py with
 * -fsanitize=address,undefined together with oracle/pkv_oracle.c.  Test infrastructure only.
 *
 * File: int64 header[24], then the arrays named below, each preceded by its int64 byte count. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int orc_paged_decode_attention(int B, int Hq, int Hkv, int D, int block_size, int num_pool_blocks,
                               int max_blocks_per_seq, int dtype, int64_t ksb, int64_t ksh, int64_t kst,
                               int64_t vsb, int64_t vsh, int64_t vst, const void* q, const void* k_pool,
                               const void* v_pool, const int32_t* block_tables, const int32_t* context_lens,
                               float scale, double* out, double* weights_out, int max_ctx);
int orc_kv_block_swap(int num_planes, int64_t block_bytes, int64_t src_plane_stride, int64_t dst_plane_stride,
                      int src_num_blocks, int dst_num_blocks, const uint8_t* src, uint8_t* dst,
                      const int32_t* mapping, int n_pairs);
int orc_kv_append(int B, int Hkv, int D, int bs, int nblk, int maxb, int eb, int64_t ksb, int64_t ksh,
                  int64_t kst, int64_t vsb, int64_t vsh, int64_t vst, const uint8_t* k_new,
                  const uint8_t* v_new, uint8_t* k_pool, uint8_t* v_pool, const int32_t* bt, const int32_t* cl);

static void* read_array(FILE* f, int64_t* nbytes) {
  if (fread(nbytes, sizeof *nbytes, 1, f) != 1 || *nbytes < 0) { fprintf(stderr, "short file\n"); exit(2); }
  void* p = malloc(*nbytes ? (size_t)*nbytes : 1);
  if (!p || fread(p, 1, (size_t)*nbytes, f) != (size_t)*nbytes) { fprintf(stderr, "short array\n"); exit(2); }
  return p;
}

static void write_array(FILE* f, const void* p, int64_t nbytes) {
  fwrite(&nbytes, sizeof nbytes, 1, f);
  fwrite(p, 1, (size_t)nbytes, f);
}

int main(int argc, char** argv) {
  if (argc != 3) { fprintf(stderr, "usage: %s case.bin result.bin\n", argv[0]); return 2; }
  FILE* in = fopen(argv[1], "rb");
  FILE* out = fopen(argv[2], "wb");
  if (!in || !out) { fprintf(stderr, "cannot open files\n"); return 2; }
  int64_t h[24];
  if (fread(h, sizeof h[0], 24, in) != 24) { fprintf(stderr, "short header\n"); return 2; }
  int64_t n[8];
  int rc = 0;
  if (h[0] == 0) {          /* attention: B Hq Hkv D bs nblk maxb dtype strides[6] scale_bits */
    void* q = read_array(in, &n[0]);
    void* k = read_array(in, &n[1]);
    void* v = read_array(in, &n[2]);
    int32_t* bt = read_array(in, &n[3]);
    int32_t* cl = read_array(in, &n[4]);
    float scale;
    uint32_t sb = (uint32_t)h[15];
    memcpy(&scale, &sb, 4);
    const int64_t on = h[1] * h[2] * h[4] * (int64_t)sizeof(double);
    double* o = malloc(on ? (size_t)on : 1);
    rc = orc_paged_decode_attention((int)h[1], (int)h[2], (int)h[3], (int)h[4], (int)h[5], (int)h[6], (int)h[7],
                                    (int)h[8], h[9], h[10], h[11], h[12], h[13], h[14], q, k, v, bt, cl, scale,
                                    o, NULL, 0);
    write_array(out, o, on);
    free(q); free(k); free(v); free(bt); free(cl); free(o);
  } else if (h[0] == 1) {   /* swap: planes block_bytes sstride dstride snb dnb npairs */
    uint8_t* src = read_array(in, &n[0]);
    uint8_t* dst = read_array(in, &n[1]);
    int32_t* mp = read_array(in, &n[2]);
    rc = orc_kv_block_swap((int)h[1], h[2], h[3], h[4], (int)h[5], (int)h[6], src, dst, mp, (int)h[7]);
    write_array(out, dst, n[1]);
    free(src); free(dst); free(mp);
  } else {                  /* append: B Hkv D bs nblk maxb eb strides[6] */
    uint8_t* kn = read_array(in, &n[0]);
    uint8_t* vn = read_array(in, &n[1]);
    uint8_t* kp = read_array(in, &n[2]);
    uint8_t* vp = read_array(in, &n[3]);
    int32_t* bt = read_array(in, &n[4]);
    int32_t* cl = read_array(in, &n[5]);
    rc = orc_kv_append((int)h[1], (int)h[2], (int)h[3], (int)h[4], (int)h[5], (int)h[6], (int)h[7], h[8], h[9],
                       h[10], h[11], h[12], h[13], kn, vn, kp, vp, bt, cl);
    write_array(out, kp, n[2]);
    write_array(out, vp, n[3]);
    free(kn); free(vn); free(kp); free(vp); free(bt); free(cl);
  }
  int64_t rc64 = rc;
  write_array(out, &rc64, sizeof rc64);
  fclose(in);
  fclose(out);
  return 0;
}
